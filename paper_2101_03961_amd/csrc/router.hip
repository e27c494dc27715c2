// Router kernels: fp32 logits, softmax, top-1, in-block ranks, per-expert scan,
// load-balancing loss, and the router's backward pass.
//
// The router is computed in fp32 whatever the activation dtype is (Sec. 2.4,
// selective precision): x is widened to fp32 before the contraction.
#include "common.h"

namespace sw {

// -----------------------------------------------------------------------------
// Logits tile kernel:  h[t][e] = sum_k x[t][k] W_r[k][e] (+ b_r[e]), fp32 FMA chain
// over k ascending (x[t][k] times its jitter multiplier when input jitter is on).
// Block = 256 tokens x 64 experts, thread = 8 tokens x 8 experts.
// -----------------------------------------------------------------------------
constexpr int kLogTB = 256;  // tokens per block
constexpr int kLogEB = 64;   // experts per block
constexpr int kLogKC = 16;   // k chunk

template <typename XT>
__global__ __launch_bounds__(256) void router_logits_kernel(const XT *__restrict__ x,
                                                            const float *__restrict__ W_r,
                                                            const float *__restrict__ b_r,
                                                            float *__restrict__ logits, int T,
                                                            int d, int E, Noise nz) {
    __shared__ float xs[kLogKC][kLogTB + 4];
    __shared__ float wsm[kLogKC][kLogEB + 4];
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * kLogTB;
    const int e0 = blockIdx.y * kLogEB;
    const int tx = tid % 8;   // expert group
    const int ty = tid / 8;   // token group
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < d; k0 += kLogKC) {
        {   // x tile: thread loads 16 consecutive k of one token, stores transposed
            const int t = t0 + tid;
#pragma unroll
            for (int kk = 0; kk < kLogKC; ++kk) {
                float v = 0.f;
                if (t < T && k0 + kk < d) {
                    v = to_f32(x[(size_t)t * d + k0 + kk]);
                    // input jitter (App. C): the router sees x * m
                    if (nz.jitter) v *= jitter_of(nz, (uint32_t)t * (uint32_t)d + (uint32_t)(k0 + kk));
                }
                xs[kk][tid] = v;
            }
        }
        {   // W tile: 16 x 64, four consecutive experts per thread
            const int kk = tid / 16;
            const int ee = (tid % 16) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = 0.f;
                if (k0 + kk < d && e0 + ee + j < E) v = W_r[(size_t)(k0 + kk) * E + e0 + ee + j];
                wsm[kk][ee + j] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kLogKC; ++kk) {
            float xv[8], wv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = xs[kk][ty * 8 + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) wv[j] = wsm[kk][tx * 8 + j];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int t = t0 + ty * 8 + i;
        if (t >= T) continue;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = e0 + tx * 8 + j;
            if (e < E) logits[(size_t)t * E + e] = acc[i][j] + (b_r ? b_r[e] : 0.f);
        }
    }
}

// -----------------------------------------------------------------------------
// Softmax / top-1 / block statistics.  Block = kRouteTB tokens, 4 waves; a wave
// walks its 64 tokens one at a time with lanes striding the experts.
// EPL = experts per lane (E <= 64 * EPL).
// -----------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// WAVES waves share the block's kRouteTB tokens (16 when the per-wave probability sums fit
// the LDS: few waves per CU leave this kernel waiting on its own loads).
template <int EPL, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void router_softmax_kernel(
    float *__restrict__ probs /* in: logits, out: p */, float *__restrict__ logits_copy,
    int32_t *__restrict__ idx_out, float *__restrict__ gate_out, int32_t *__restrict__ idx_ws,
    float *__restrict__ gate_ws, int32_t *__restrict__ local_rank,
    int32_t *__restrict__ block_counts, float *__restrict__ block_psum, int nbg, int Tg, int E) {
    extern __shared__ char smem_raw[];
    // layout: idx_s[kRouteTB] | hist[E] | psum_w[WAVES][E]
    int32_t *idx_s = (int32_t *)smem_raw;
    int32_t *hist = idx_s + kRouteTB;
    float *psum_w = (float *)(hist + E);

    const int tid = threadIdx.x;
    const int lane = tid % kWave;
    const int wave = tid / kWave;
    const int b = blockIdx.x;
    int t0, tend;
    block_token_range(b, nbg, Tg, t0, tend);
    constexpr int kThreads = WAVES * kWave;
    constexpr int kTokPerWave = kRouteTB / WAVES;
    for (int e = tid; e < E; e += kThreads) hist[e] = 0;

    float pacc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) pacc[j] = 0.f;

    // kU tokens at a time (their loads and reductions overlap); every token's arithmetic, and the
    // order in which the tokens enter the probability sums, is that of a one-by-one walk
    constexpr int kU = EPL <= 4 ? 4 : (EPL <= 8 ? 2 : 1);
    static_assert(kTokPerWave % kU == 0, "tokens per wave");
    for (int i0 = 0; i0 < kTokPerWave; i0 += kU) {
        float h[kU][EPL], best[kU], z[kU];
        int besti[kU];
        bool live[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int t = t0 + wave * kTokPerWave + i0 + u;
            live[u] = t < tend;
            best[u] = -INFINITY;
            besti[u] = 0x7fffffff;
            const float *row = probs + (size_t)(live[u] ? t : t0) * E;
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const int e = lane + j * kWave;
                h[u][j] = (live[u] && e < E) ? row[e] : -INFINITY;
                if (h[u][j] > best[u]) { best[u] = h[u][j]; besti[u] = e; }   // ascending e: lowest index kept on ties
            }
        }
        if (logits_copy) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int j = 0; j < EPL; ++j) {
                    const int e = lane + j * kWave;
                    if (live[u] && e < E)
                        logits_copy[(size_t)(t0 + wave * kTokPerWave + i0 + u) * E + e] = h[u][j];
                }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1)
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const float ov = __shfl_xor(best[u], m, kWave);
                const int oi = __shfl_xor(besti[u], m, kWave);
                if (ov > best[u] || (ov == best[u] && oi < besti[u])) { best[u] = ov; besti[u] = oi; }
            }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            z[u] = 0.f;
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const int e = lane + j * kWave;
                // the hardware exp2 is accurate to about one ulp, the scaled argument adds
                // |h - best| 2^-24: far inside the 1e-5 budget
                h[u][j] = (live[u] && e < E) ? __expf(h[u][j] - best[u]) : 0.f;
                z[u] += h[u][j];
            }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1)
#pragma unroll
            for (int u = 0; u < kU; ++u) z[u] += __shfl_xor(z[u], m, kWave);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int tl = wave * kTokPerWave + i0 + u;
            const int t = t0 + tl;
            if (!live[u]) {
                if (lane == 0) idx_s[tl] = -1;
                continue;
            }
            float *row = probs + (size_t)t * E;
            const float g = 1.0f / z[u];   // exp(0) / z: also the probability of the arg max
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const int e = lane + j * kWave;
                const float p = h[u][j] * g;
                if (e < E) row[e] = p;
                pacc[j] += p;   // padded experts add 0
            }
            if (lane == 0) {
                idx_s[tl] = besti[u];
                idx_out[t] = besti[u];
                idx_ws[t] = besti[u];
                gate_out[t] = g;
                gate_ws[t] = g;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
        const int e = lane + j * kWave;
        if (e < E) psum_w[wave * E + e] = pacc[j];
    }
    __syncthreads();
    // rank of each token among the block's earlier tokens with the same expert
    if (tid < kRouteTB) {
        const int me = idx_s[tid];
        if (me >= 0) {
            int r = 0;
            for (int s = 0; s < tid; ++s) r += (idx_s[s] == me);
            local_rank[t0 + tid] = r;
            atomicAdd(&hist[me], 1);   // integer: result independent of order
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += kThreads) {
        block_counts[(size_t)b * E + e] = hist[e];
        float ps = psum_w[e];   // fixed order over the waves
#pragma unroll
        for (int q = 1; q < WAVES; ++q) ps += psum_w[q * E + e];
        block_psum[(size_t)b * E + e] = ps;
    }
}

// -----------------------------------------------------------------------------
// Per-expert scan over token blocks: each block of 1024 threads takes a slice of the experts
// and leaves its part of sum_e (counts / T) (psum / T) in loss_part; positions_kernel adds
// the parts up in block order.
//   block_off[b][e] = sum_{b' < b} block_counts[b'][e]
//   counts[e], kept[e] = min(counts[e], C),  P-sum[e] in fixed order
//   aux = alpha * E * sum_e (counts[e] / T) * (psum[e] / T)             (Eqs. 4-6)
// -----------------------------------------------------------------------------
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void route_scan_kernel(
    const int32_t *__restrict__ block_counts, const float *__restrict__ block_psum,
    int32_t *__restrict__ block_off, int32_t *__restrict__ counts_ws, int32_t *__restrict__ kept_ws,
    int32_t *__restrict__ counts_g, int32_t *__restrict__ grp_off, int32_t *__restrict__ counts_out,
    double *__restrict__ loss_part, uint32_t *__restrict__ slot_off, int slot_off_n, int nb, int E,
    int C, int T) {
    // every slot starts without a token (the position kernel, which runs next, fills in the rest)
    for (int i = blockIdx.x * kScanThreads + threadIdx.x; i < slot_off_n; i += gridDim.x * kScanThreads)
        slot_off[i] = kNoRow;
    __shared__ int32_t part_cnt[kScanThreads];
    __shared__ float part_ps[kScanThreads];
    __shared__ double red[kScanThreads];
    const int tid = threadIdx.x;
    // this block's experts: [e_lo, e_hi)
    const int slice = (E + (int)gridDim.x - 1) / (int)gridDim.x;
    const int e_lo = blockIdx.x * slice;
    const int e_hi = e_lo + slice < E ? e_lo + slice : E;
    const int Ew = slice < kScanThreads ? slice : kScanThreads;   // experts handled per pass
    const int P = kScanThreads / Ew;                              // block-range parts per expert
    const int el = tid % Ew;
    const int part = tid / Ew;
    const int per = (nb + P - 1) / P;
    const int b_lo = part * per;
    const int b_hi = (b_lo + per < nb) ? b_lo + per : nb;
    double loss_acc = 0.0;
    for (int ebase = e_lo; ebase < e_hi; ebase += Ew) {
        const int e = ebase + el;
        const bool active = part < P && e < e_hi;
        int csum = 0;
        float psum = 0.f;
        if (active)
            for (int b = b_lo; b < b_hi; ++b) {
                csum += block_counts[(size_t)b * E + e];
                psum += block_psum[(size_t)b * E + e];
            }
        part_cnt[tid] = csum;
        part_ps[tid] = psum;
        __syncthreads();
        int start = 0;
        if (active) {
            for (int q = 0; q < part; ++q) start += part_cnt[q * Ew + el];
            int run = start;
            for (int b = b_lo; b < b_hi; ++b) {
                block_off[(size_t)b * E + e] = run;
                run += block_counts[(size_t)b * E + e];
            }
        }
        if (part == 0 && e < e_hi) {
            int total = 0;
            float ptot = 0.f;
            for (int q = 0; q < P; ++q) {
                total += part_cnt[q * Ew + el];
                ptot += part_ps[q * Ew + el];
            }
            counts_ws[e] = total;
            counts_g[e] = total;   // one group
            grp_off[e] = 0;
            counts_out[e] = total;
            kept_ws[e] = total < C ? total : C;
            loss_acc += ((double)total / (double)T) * ((double)ptot / (double)T);
        }
        __syncthreads();
    }
    red[tid] = loss_acc;
    __syncthreads();
    for (int s = kScanThreads / 2; s >= 1; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) loss_part[blockIdx.x] = red[0];
}

// -----------------------------------------------------------------------------
// The same for several routing groups (single block).  Phase 1, one thread per (group,
// expert) pair: exclusive scan of the group's blocks, counts_g and P-sums.  Phase 2, one
// thread per expert: slots of the groups inside the expert's buffer (grp_off), totals, and the
// expert's share of   aux = (1/n) sum_g alpha E sum_e (counts_g / Tg) (psum_g / Tg).
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(kScanThreads) void route_scan_groups_kernel(
    const int32_t *__restrict__ block_counts, const float *__restrict__ block_psum,
    int32_t *__restrict__ block_off, int32_t *__restrict__ counts_ws, int32_t *__restrict__ kept_ws,
    int32_t *__restrict__ counts_g, float *__restrict__ psum_g, int32_t *__restrict__ grp_off,
    int32_t *__restrict__ counts_out, double *__restrict__ loss_part,
    uint32_t *__restrict__ slot_off, int slot_off_n, int n, int nbg, int E, int Cg, int Tg) {
    __shared__ double red[kScanThreads];
    const int tid = threadIdx.x;
    for (int i = tid; i < slot_off_n; i += kScanThreads) slot_off[i] = kNoRow;
    for (int pair = tid; pair < n * E; pair += kScanThreads) {
        const int g = pair / E, e = pair - g * E;
        int run = 0;
        float ps = 0.f;
        for (int b = g * nbg; b < (g + 1) * nbg; ++b) {
            block_off[(size_t)b * E + e] = run;
            run += block_counts[(size_t)b * E + e];
            ps += block_psum[(size_t)b * E + e];
        }
        counts_g[pair] = run;
        psum_g[pair] = ps;
    }
    __syncthreads();   // the block's own global writes are visible to it after the barrier
    double loss_acc = 0.0;
    for (int e = tid; e < E; e += kScanThreads) {
        int total = 0, kept = 0;
        for (int g = 0; g < n; ++g) {
            const int c = counts_g[g * E + e];
            grp_off[g * E + e] = kept;
            kept += c < Cg ? c : Cg;
            total += c;
            loss_acc += ((double)c / (double)Tg) * ((double)psum_g[g * E + e] / (double)Tg);
        }
        counts_ws[e] = total;
        counts_out[e] = total;
        kept_ws[e] = kept;
    }
    red[tid] = loss_acc;
    __syncthreads();
    for (int s = kScanThreads / 2; s >= 1; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) loss_part[0] = red[0];
}

// -----------------------------------------------------------------------------
// Backward, step 1: gradient w.r.t. the logits.
//   dp[t][i] = dgate[t] [i = e_t] + d_aux * alpha * E * (counts_g[g][i] / Tg) / (n Tg),  t in group g
//              (evaluated with counts_g - Tg / E: a constant shift of dp leaves dl unchanged)
//   dl[t][j] = p[t][j] (dp[t][j] - sum_i p[t][i] dp[t][i])
// One wave per token, lanes stride the experts.
// -----------------------------------------------------------------------------
// tokens a wave works on at once (their loads overlap); one when the experts fill the registers
constexpr int dl_tokens(int epl) { return epl <= 4 ? 4 : 1; }

template <int EPL>
__global__ __launch_bounds__(256) void router_dlogits_kernel(
    const float *__restrict__ probs, const int32_t *__restrict__ idx,
    const float *__restrict__ dgate, const int32_t *__restrict__ counts_g /* [n][E] */,
    float *__restrict__ dlogits /* [T][E] or nullptr */,
    bf16 *__restrict__ dl_split /* [T][256] hi | lo, or nullptr */,
    int T, int Tg, int E, float aux_scale /* d_aux*alpha*E/(n Tg^2) */) {
    constexpr int kDlTokens = dl_tokens(EPL);
    const int epad = (E + 127) / 128 * 128;
    const float mean_count = (float)Tg / (float)E;
    const int lane = threadIdx.x % kWave;
    const int t_first = (blockIdx.x * (256 / kWave) + threadIdx.x / kWave) * kDlTokens;
    float p[kDlTokens][EPL], dp[kDlTokens][EPL], s[kDlTokens];
#pragma unroll
    for (int u = 0; u < kDlTokens; ++u) {
        const int t = t_first + u;
        s[u] = 0.f;
        if (t >= T) continue;
        const int me = idx[t];
        const float dg = dgate[t];
        const int32_t *counts = counts_g + (size_t)(t / Tg) * E;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int e = lane + j * kWave;
            p[u][j] = e < E ? probs[(size_t)t * E + e] : 0.f;
            // counts enter centred on their mean Tg / E: the softmax backward subtracts the
            // p-weighted mean of dp anyway (sum_i p_i = 1), and nearly equal counts would
            // otherwise cancel to a few fp32 digits in dp - s
            dp[u][j] = e < E ? aux_scale * ((float)counts[e] - mean_count) : 0.f;
            if (e == me) dp[u][j] += dg;
            s[u] += p[u][j] * dp[u][j];
        }
    }
#pragma unroll
    for (int u = 0; u < kDlTokens; ++u) s[u] = wave_sum(s[u]);
#pragma unroll
    for (int u = 0; u < kDlTokens; ++u) {
        const int t = t_first + u;
        if (t >= T) continue;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int e = lane + j * kWave;
            const float dl = e < E ? p[u][j] * (dp[u][j] - s[u]) : 0.f;
            if (dlogits && e < E) dlogits[(size_t)t * E + e] = dl;
            if (dl_split && e < epad) {   // two bf16 terms (16 mantissa bits) for the MFMA contractions,
                const bf16 hi = (bf16)dl;  // one [T][hi 128 | lo 128] plane per tile of 128 experts
                bf16 *row = dl_split + ((size_t)(e >> 7) * T + t) * 256 + (e & 127);
                row[0] = hi;
                row[128] = (bf16)(dl - (float)hi);
            }
        }
        if (dl_split)   // columns of the 128-wide halves that no lane visited above
            for (int e = lane + EPL * kWave; e < epad; e += kWave) {
                bf16 *row = dl_split + ((size_t)(e >> 7) * T + t) * 256 + (e & 127);
                row[0] = (bf16)0.f;
                row[128] = (bf16)0.f;
            }
    }
}

// The same for the matrix-core backward (E <= 128, E % 4 == 0): a lane owns the two adjacent
// experts 2 lane and 2 lane + 1, so a wave reads a probability row with one 8-byte load per
// lane and writes the bf16 hi | lo halves as 4-byte pairs; four tokens per wave at once.
__global__ __launch_bounds__(256) void router_dlogits_pair_kernel(
    const float *__restrict__ probs, const int32_t *__restrict__ idx,
    const float *__restrict__ dgate, const int32_t *__restrict__ counts_g /* [n][E] */,
    float *__restrict__ dlogits /* [T][E] or nullptr */, bf16 *__restrict__ dl_split /* [T][256] */,
    int T, int Tg, int E, float aux_scale) {
    typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
    constexpr int kTok = 4;
    const float mean_count = (float)Tg / (float)E;
    const int lane = threadIdx.x % kWave;
    const int t_first = (blockIdx.x * (256 / kWave) + threadIdx.x / kWave) * kTok;
    const int e0 = 2 * lane;
    const bool live = e0 < E;   // E is even: both experts of the lane or neither
    float2 p[kTok], dp[kTok];
    float s[kTok];
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int t = t_first + u;
        s[u] = 0.f;
        p[u] = dp[u] = make_float2(0.f, 0.f);
        if (t >= T || !live) continue;
        const int me = idx[t];
        const float dg = dgate[t];
        const int2 c = *(const int2 *)(counts_g + (size_t)(t / Tg) * E + e0);
        p[u] = *(const float2 *)(probs + (size_t)t * E + e0);
        dp[u].x = aux_scale * ((float)c.x - mean_count) + (me == e0 ? dg : 0.f);
        dp[u].y = aux_scale * ((float)c.y - mean_count) + (me == e0 + 1 ? dg : 0.f);
        s[u] = p[u].x * dp[u].x + p[u].y * dp[u].y;
    }
#pragma unroll
    for (int u = 0; u < kTok; ++u) s[u] = wave_sum(s[u]);
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int t = t_first + u;
        if (t >= T) continue;
        const float2 dl = make_float2(p[u].x * (dp[u].x - s[u]), p[u].y * (dp[u].y - s[u]));   // 0 past E
        if (dlogits && live) *(float2 *)(dlogits + (size_t)t * E + e0) = dl;
        bf16x2 hi, lo;
        hi[0] = (bf16)dl.x;
        hi[1] = (bf16)dl.y;
        lo[0] = (bf16)(dl.x - (float)hi[0]);
        lo[1] = (bf16)(dl.y - (float)hi[1]);
        *(bf16x2 *)(dl_split + (size_t)t * 256 + e0) = hi;        // all 128 columns of each half
        *(bf16x2 *)(dl_split + (size_t)t * 256 + 128 + e0) = lo;
    }
}

// dW_r[k][j] = sum over splits of (part[s][k][j] + part[s][k][128 + j]), fixed order.
// rows = rows of one split's part; second > 0: the operand had a second plane (input jitter:
// x * m as hi + mid), whose rows start at `second` and are added in.
__global__ __launch_bounds__(256) void reduce_dWr_split_kernel(const float *__restrict__ part,
                                                               float *__restrict__ dW_r, int d,
                                                               int E, int nsplit, int rows,
                                                               int second) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= d * E) return;
    const int k = i / E, j = i - k * E;
    // the parts of expert j's tile of 128 experts: [tile][split][rows][hi 128 | lo 128]
    const float *tile_part = part + (size_t)(j >> 7) * nsplit * rows * 256 + (j & 127);
    float s = 0.f;
#pragma unroll 8
    for (int q = 0; q < nsplit; ++q) {   // unrolled: eight splits' loads in flight, same order of sums
        const float *row = tile_part + ((size_t)q * rows + k) * 256;
        s += row[0] + row[128];
    }
    if (second > 0) {
        float s2 = 0.f;
#pragma unroll 8
        for (int q = 0; q < nsplit; ++q) {
            const float *row = tile_part + ((size_t)q * rows + second + k) * 256;
            s2 += row[0] + row[128];
        }
        s += s2;
    }
    dW_r[i] = s;
}

// Input jitter with the matrix-core router backward: dx holds the router's product
// dl W_r^T (rounded to bf16); finish  dx[t][k] = m[t][k] * dx[t][k] + dXd[slot_t][k].
__global__ __launch_bounds__(256) void router_dx_jitter_kernel(bf16 *__restrict__ dx,
                                                               const bf16 *__restrict__ dXd,
                                                               const int32_t *__restrict__ tok_slot,
                                                               int T, int d, Noise nz) {
    typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
    const int cpr = d / 8;
    const long chunk = (long)blockIdx.x * 256 + threadIdx.x;
    if (chunk >= (long)T * cpr) return;
    const int t = (int)(chunk / cpr);
    const int k0 = (int)(chunk - (long)t * cpr) * 8;
    bf16x8 v = *(const bf16x8 *)(dx + (size_t)t * d + k0);
    const int slot = tok_slot[t];
    bf16x8 add;
    if (slot >= 0) add = *(const bf16x8 *)(dXd + (size_t)slot * d + k0);
    const uint32_t idx = (uint32_t)t * (uint32_t)d + (uint32_t)k0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float r = (float)v[i] * jitter_of(nz, idx + (uint32_t)i);
        if (slot >= 0) r += (float)add[i];
        v[i] = (bf16)r;
    }
    *(bf16x8 *)(dx + (size_t)t * d + k0) = v;
}

// 4-byte words set to -1
__global__ __launch_bounds__(256) void fill_minus_one_kernel(int32_t *__restrict__ p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = -1;
}

// -----------------------------------------------------------------------------
// Backward, step 2:  dx[t][k] = m[t][k] sum_j dl[t][j] W_r[k][j] + kept_t * dXd[slot_t][k]
// (m: the jitter multiplier the router's input carried, 1 without jitter)
// Block = 256 tokens x 64 k, thread = 8 tokens x 8 k, reduction over experts.
// -----------------------------------------------------------------------------
template <typename XT>
__global__ __launch_bounds__(256) void router_dx_kernel(
    const float *__restrict__ dlogits, const float *__restrict__ W_r,
    const XT *__restrict__ dXd, const int32_t *__restrict__ tok_slot, XT *__restrict__ dx, int T,
    int d, int E, Noise nz) {
    __shared__ float ds[kLogKC][kLogTB + 4];
    __shared__ float wsm[kLogKC][kLogEB + 4];
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * kLogTB;
    const int k0 = blockIdx.y * kLogEB;
    const int tx = tid % 8, ty = tid / 8;
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int j0 = 0; j0 < E; j0 += kLogKC) {
        {
            const int t = t0 + tid;
#pragma unroll
            for (int jj = 0; jj < kLogKC; ++jj) {
                float v = 0.f;
                if (t < T && j0 + jj < E) v = dlogits[(size_t)t * E + j0 + jj];
                ds[jj][tid] = v;
            }
        }
        {   // W_r[k][j] -> wsm[jj][kk]; thread reads 4 consecutive j of one k
            const int kk = tid / 4;            // 0..63
            const int jq = (tid % 4) * 4;      // 0,4,8,12
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float v = 0.f;
                if (k0 + kk < d && j0 + jq + u < E) v = W_r[(size_t)(k0 + kk) * E + j0 + jq + u];
                wsm[jq + u][kk] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < kLogKC; ++jj) {
            float dv[8], wv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) dv[i] = ds[jj][ty * 8 + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) wv[j] = wsm[jj][tx * 8 + j];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(dv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int t = t0 + ty * 8 + i;
        if (t >= T) continue;
        const int slot_or_none = tok_slot[t];
        const bool kept = slot_or_none >= 0;
        const size_t slot = kept ? (size_t)slot_or_none : 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = k0 + tx * 8 + j;
            if (k >= d) continue;
            float v = acc[i][j];
            if (nz.jitter) v *= jitter_of(nz, (uint32_t)t * (uint32_t)d + (uint32_t)k);
            if (kept) v += to_f32(dXd[slot * d + k]);
            dx[(size_t)t * d + k] = from_f32<XT>(v);
        }
    }
}

// -----------------------------------------------------------------------------
// Backward, step 3:  dW_r[k][j] = sum_t x[t][k] dl[t][j] (x times its jitter multiplier
// when input jitter is on), split over token ranges.
// Block = 64 k x 64 j output tile over one token range; thread = 4 k x 4 j.
// Partial sums are combined in split order by reduce_partials_kernel, so the
// result does not depend on scheduling.
// -----------------------------------------------------------------------------
constexpr int kWrTile = 64;
constexpr int kWrTC = 16;

template <typename XT>
__global__ __launch_bounds__(256) void router_dWr_kernel(const XT *__restrict__ x,
                                                         const float *__restrict__ dlogits,
                                                         float *__restrict__ part, int T, int d,
                                                         int E, int tokens_per_split, Noise nz) {
    __shared__ float xs[kWrTC][kWrTile + 4];
    __shared__ float ls[kWrTC][kWrTile + 4];
    const int tid = threadIdx.x;
    const int k0 = blockIdx.x * kWrTile;
    const int j0 = blockIdx.y * kWrTile;
    const int split = blockIdx.z;
    const int t_lo = split * tokens_per_split;
    const int t_hi = (t_lo + tokens_per_split < T) ? t_lo + tokens_per_split : T;
    const int tx = tid % 16, ty = tid / 16;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int tb = t_lo; tb < t_hi; tb += kWrTC) {
        {
            const int tt = tid / 16;          // 0..15 token within chunk
            const int cc = (tid % 16) * 4;    // 4 consecutive columns
            const int t = tb + tt;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float xv = 0.f, lv = 0.f;
                if (t < t_hi) {
                    if (k0 + cc + u < d) {
                        xv = to_f32(x[(size_t)t * d + k0 + cc + u]);
                        if (nz.jitter)
                            xv *= jitter_of(nz, (uint32_t)t * (uint32_t)d + (uint32_t)(k0 + cc + u));
                    }
                    if (j0 + cc + u < E) lv = dlogits[(size_t)t * E + j0 + cc + u];
                }
                xs[tt][cc + u] = xv;
                ls[tt][cc + u] = lv;
            }
        }
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < kWrTC; ++tt) {
            float xv[4], lv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = xs[tt][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) lv[j] = ls[tt][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], lv[j], acc[i][j]);
        }
        __syncthreads();
    }
    float *out = part + (size_t)split * d * E;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = k0 + ty * 4 + i;
        if (k >= d) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = j0 + tx * 4 + j;
            if (e < E) out[(size_t)k * E + e] = acc[i][j];
        }
    }
}

// db_r partials: part[split][j] = sum over the split's tokens of dl[t][j]
__global__ __launch_bounds__(256) void router_dbr_kernel(const float *__restrict__ dlogits,
                                                         float *__restrict__ part, int T, int E) {
    // one block per 256 tokens; a thread sums a column in four interleaved chains (fixed order)
    const int t_lo = blockIdx.x * 256;
    const int t_hi = (t_lo + 256 < T) ? t_lo + 256 : T;
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int t = t_lo;
        for (; t + 3 < t_hi; t += 4) {
            s0 += dlogits[(size_t)t * E + e];
            s1 += dlogits[(size_t)(t + 1) * E + e];
            s2 += dlogits[(size_t)(t + 2) * E + e];
            s3 += dlogits[(size_t)(t + 3) * E + e];
        }
        for (; t < t_hi; ++t) s0 += dlogits[(size_t)t * E + e];
        part[(size_t)blockIdx.x * E + e] = (s0 + s1) + (s2 + s3);
    }
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part,
                                                              float *__restrict__ out, size_t n,
                                                              int nsplit) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
#pragma unroll 8
    for (int q = 0; q < nsplit; ++q) s += part[(size_t)q * n + i];
    out[i] = s;
}

// -----------------------------------------------------------------------------
// launchers
// -----------------------------------------------------------------------------
template <int EPL>
static hipError_t softmax_launch(const Workspace &w, char *ws, int32_t *expert_index, float *gate,
                                 float *router_logits, hipStream_t s) {
    constexpr int kWaves = EPL <= 8 ? 16 : 4;   // 16 x 512 experts x 4 bytes = 32 KB of sums at most
    const size_t smem = sizeof(int32_t) * kRouteTB + sizeof(int32_t) * w.E + sizeof(float) * kWaves * w.E;
    hipLaunchKernelGGL((router_softmax_kernel<EPL, kWaves>), dim3((unsigned)w.nb), dim3(kWaves * kWave),
                       smem, s, (float *)(ws + w.probs), router_logits, expert_index, gate,
                       (int32_t *)(ws + w.idx), (float *)(ws + w.gate),
                       (int32_t *)(ws + w.local_rank), (int32_t *)(ws + w.block_counts),
                       (float *)(ws + w.block_psum), (int)w.nbg, (int)w.Tg, (int)w.E);
    return hipGetLastError();
}

#define SW_DISPATCH_EPL(E, CALL)                  \
    do {                                          \
        if ((E) <= 64) { CALL(1); }               \
        else if ((E) <= 128) { CALL(2); }         \
        else if ((E) <= 256) { CALL(4); }         \
        else if ((E) <= 512) { CALL(8); }         \
        else if ((E) <= 1024) { CALL(16); }       \
        else if ((E) <= 2048) { CALL(32); }       \
        else { CALL(64); }                        \
    } while (0)

hipError_t launch_router_fwd(const Workspace &w, int dtype, const void *x, const float *W_r,
                             const float *b_r, char *ws, int32_t *expert_index, float *gate,
                             float *router_logits, hipStream_t s) {
    hipError_t err;
    {
        ProfScope ps("router_logits", s);
        dim3 grid((unsigned)ceil_div(w.T, kLogTB), (unsigned)ceil_div(w.E, kLogEB));
        if (dtype == SW_BF16)
            hipLaunchKernelGGL(router_logits_kernel<bf16>, grid, dim3(256), 0, s, (const bf16 *)x,
                               W_r, b_r, (float *)(ws + w.probs), (int)w.T, (int)w.d, (int)w.E,
                               w.noise);
        else
            hipLaunchKernelGGL(router_logits_kernel<float>, grid, dim3(256), 0, s,
                               (const float *)x, W_r, b_r, (float *)(ws + w.probs), (int)w.T,
                               (int)w.d, (int)w.E, w.noise);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    return launch_router_softmax(w, ws, expert_index, gate, router_logits, s);
}

hipError_t launch_router_softmax(const Workspace &w, char *ws, int32_t *expert_index, float *gate,
                                 float *router_logits, hipStream_t s) {
    hipError_t err = hipSuccess;
    ProfScope ps("router_softmax_top1", s);
#define CALL(N) err = softmax_launch<N>(w, ws, expert_index, gate, router_logits, s)
    SW_DISPATCH_EPL(w.E, CALL);
#undef CALL
    return err;
}

int route_scan_blocks(const Workspace &w) {
    if (w.n > 1) return 1;
    return w.E >= 64 ? 8 : 1;
}

hipError_t launch_route_scan(const Workspace &w, char *ws, int32_t *expert_counts, hipStream_t s) {
    ProfScope ps("route_scan_aux", s);
    if (w.n == 1)
        hipLaunchKernelGGL(route_scan_kernel, dim3((unsigned)route_scan_blocks(w)),
                           dim3(kScanThreads), 0, s, (const int32_t *)(ws + w.block_counts),
                           (const float *)(ws + w.block_psum), (int32_t *)(ws + w.block_off),
                           (int32_t *)(ws + w.counts), (int32_t *)(ws + w.kept),
                           (int32_t *)(ws + w.counts_g), (int32_t *)(ws + w.grp_off),
                           expert_counts, (double *)(ws + w.loss_part),
                           (uint32_t *)(ws + w.slot_off), (int)(w.E * w.C + 128), (int)w.nb,
                           (int)w.E, (int)w.C, (int)w.T);
    else
        hipLaunchKernelGGL(route_scan_groups_kernel, dim3(1), dim3(kScanThreads), 0, s,
                           (const int32_t *)(ws + w.block_counts),
                           (const float *)(ws + w.block_psum), (int32_t *)(ws + w.block_off),
                           (int32_t *)(ws + w.counts), (int32_t *)(ws + w.kept),
                           (int32_t *)(ws + w.counts_g), (float *)(ws + w.psum_g),
                           (int32_t *)(ws + w.grp_off), expert_counts,
                           (double *)(ws + w.loss_part), (uint32_t *)(ws + w.slot_off),
                           (int)(w.E * w.C + 128), (int)w.n, (int)w.nbg, (int)w.E, (int)w.Cg,
                           (int)w.Tg);
    return hipGetLastError();
}

template <typename XT>
static hipError_t router_bwd_typed(const Workspace &w, float alpha, float d_aux, const XT *x,
                                   const float *W_r, char *ws, XT *dx, float *dW_r, float *db_r,
                                   hipStream_t s) {
    hipError_t err = hipSuccess;
    float *dlogits = (float *)(ws + w.dlogits);
    // bf16 tokens and up to 128 experts: the two contractions run on the matrix cores
    // (dl and W_r as two bf16 terms each; x is bf16 already)
    // (the forward pass took the same path and left W_r's bf16 terms in the workspace)
    const bool mfma = router_bwd_mfma_supported(w, sizeof(XT) == 2 ? SW_BF16 : SW_F32);
    bf16 *dl_split = mfma ? (bf16 *)(ws + w.dl_split) : nullptr;
    // the fp32 copy is read only by the vector-ALU contractions and by the bias gradient
    float *dlogits_out = (mfma && !db_r) ? nullptr : dlogits;
    {
        ProfScope ps("router_dlogits", s);
        const float aux_scale = (float)((double)d_aux * (double)alpha * (double)w.E /
                                        ((double)w.n * (double)w.Tg * (double)w.Tg));
#define CALL(N)                                                                                  \
    hipLaunchKernelGGL(router_dlogits_kernel<N>,                                                  \
                       dim3((unsigned)ceil_div(w.T, 4 * dl_tokens(N))), dim3(256), 0,             \
                       s, (const float *)(ws + w.probs), (const int32_t *)(ws + w.idx),          \
                       (const float *)(ws + w.dgate), (const int32_t *)(ws + w.counts_g),        \
                       dlogits_out, dl_split, (int)w.T, (int)w.Tg, (int)w.E, aux_scale)
        if (mfma && w.etiles == 1)
            hipLaunchKernelGGL(router_dlogits_pair_kernel, dim3((unsigned)ceil_div(w.T, 16)), dim3(256),
                               0, s, (const float *)(ws + w.probs), (const int32_t *)(ws + w.idx),
                               (const float *)(ws + w.dgate), (const int32_t *)(ws + w.counts_g),
                               dlogits_out, dl_split, (int)w.T, (int)w.Tg, (int)w.E, aux_scale);
        else
            SW_DISPATCH_EPL(w.E, CALL);
#undef CALL
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (mfma) {
        const bool jitter = w.noise.jitter;
        if (jitter) {   // the matrix-core kernel writes the bare product: no token has an addend
            hipLaunchKernelGGL(fill_minus_one_kernel, dim3((unsigned)ceil_div(w.T, 256)), dim3(256),
                               0, s, (int32_t *)(ws + w.no_slot), (int)w.T);
            if ((err = hipGetLastError()) != hipSuccess) return err;
        }
        if ((err = launch_router_dx_mfma(w, ws, dx, s)) != hipSuccess) return err;
        if (jitter) {
            ProfScope ps("router_dx_jitter", s);
            const long chunks = (long)w.T * (w.d / 8);
            hipLaunchKernelGGL(router_dx_jitter_kernel, dim3((unsigned)ceil_div(chunks, 256)),
                               dim3(256), 0, s, (bf16 *)dx, (const bf16 *)(ws + w.dXd),
                               (const int32_t *)(ws + w.tok_slot), (int)w.T, (int)w.d, w.noise);
            if ((err = hipGetLastError()) != hipSuccess) return err;
        }
        if ((err = launch_router_dWr_mfma(w, x, ws, s)) != hipSuccess) return err;
        ProfScope ps("router_dWr_reduce", s);
        hipLaunchKernelGGL(reduce_dWr_split_kernel, dim3((unsigned)ceil_div(w.d * w.E, 256)),
                           dim3(256), 0, s, (const float *)(ws + w.dWr_part_m), dW_r, (int)w.d,
                           (int)w.E, (int)w.nsplit_m, jitter ? 2 * (int)w.dpad : (int)w.d,
                           jitter ? (int)w.dpad : 0);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    } else {
        ProfScope ps("router_dx", s);
        dim3 grid((unsigned)ceil_div(w.T, kLogTB), (unsigned)ceil_div(w.d, kLogEB));
        hipLaunchKernelGGL(router_dx_kernel<XT>, grid, dim3(256), 0, s, dlogits, W_r,
                           (const XT *)(ws + w.dXd), (const int32_t *)(ws + w.tok_slot), dx,
                           (int)w.T, (int)w.d, (int)w.E, w.noise);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    const int tokens_per_split = (int)ceil_div(w.T, w.nsplit);
    if (!mfma) {
        ProfScope ps("router_dWr", s);
        dim3 grid((unsigned)ceil_div(w.d, kWrTile), (unsigned)ceil_div(w.E, kWrTile),
                  (unsigned)w.nsplit);
        hipLaunchKernelGGL(router_dWr_kernel<XT>, grid, dim3(256), 0, s, x, dlogits,
                           (float *)(ws + w.dWr_part), (int)w.T, (int)w.d, (int)w.E,
                           tokens_per_split, w.noise);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        const size_t n = (size_t)w.d * w.E;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0,
                           s, (const float *)(ws + w.dWr_part), dW_r, n, (int)w.nsplit);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (db_r) {
        ProfScope ps("router_dbr", s);
        const int nblk = (int)ceil_div(w.T, 256);
        hipLaunchKernelGGL(router_dbr_kernel, dim3((unsigned)nblk), dim3(256), 0, s, dlogits,
                           (float *)(ws + w.dbr_part), (int)w.T, (int)w.E);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(w.E, 256)), dim3(256),
                           0, s, (const float *)(ws + w.dbr_part), db_r, (size_t)w.E, nblk);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    return err;
}

hipError_t launch_router_bwd(const Workspace &w, int dtype, float alpha, float d_aux,
                             const void *x, const float *W_r, char *ws, void *dx, float *dW_r,
                             float *db_r, hipStream_t s) {
    if (dtype == SW_BF16)
        return router_bwd_typed<bf16>(w, alpha, d_aux, (const bf16 *)x, W_r, ws, (bf16 *)dx, dW_r,
                                      db_r, s);
    return router_bwd_typed<float>(w, alpha, d_aux, (const float *)x, W_r, ws, (float *)dx, dW_r,
                                   db_r, s);
}

}  // namespace sw
