// No-Token-Left-Behind (App. B): re-routing stages after the Switch routing.
//
// After stage 1 (arg max routing, capacity cut) every further stage lets the tokens that are
// still without a slot ask their next-best expert -- experts ranked by logit, highest first,
// equal logits by lower index -- and hands out that expert's remaining capacity in sequence
// order inside the routing group.  A stage is the stage-1 machinery once more, on the
// stage's candidates only:
//   ntlb_choice      the expert each waiting token asks for
//   ntlb_rank        per 256-token block: a candidate's rank among the block's earlier
//                    candidates for the same expert, block histogram
//   ntlb_block_scan  per (group, expert): exclusive prefix of the histograms over the blocks
//   ntlb_expert_scan per expert: capacity still free per group, where the stage's tokens go in
//                    the expert's slot range (behind everything placed before), new totals
//   ntlb_place       per token: slot, tables, and the outputs of the tokens that found one
// All integer work except the comparison of fp32 logits; deterministic.
#include "common.h"

namespace sw {

// -----------------------------------------------------------------------------
// The expert each waiting token asks for.  Tokens without a slot sit at the end of their
// group's sequence (they are the ones whose rank passed the capacity), so a wave does not
// own consecutive tokens but every W-th one (W = number of waves): lane k looks at token
// k W + w, and the waiting tokens spread evenly over the waves.  A wave then visits its waiting
// tokens four at a time (their row loads overlap): the lanes stride the experts and the wave
// reduces to the best expert ranking strictly after the one asked last.
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ntlb_choice_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ tok_slot,
    const int32_t *__restrict__ first_choice, int32_t *__restrict__ asked, int T, int E, int W,
    int round) {
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= W) return;
    const long tl_ = (long)lane * W + w;
    const int tw = tl_ < T ? (int)tl_ : -1;
    const bool unplaced = tw >= 0 && tok_slot[tw] < 0;
    const int last = unplaced ? (round == 0 ? first_choice[tw] : asked[tw]) : -1;
    const float last_h = last >= 0 ? logits[(size_t)tw * E + last] : 0.f;
    int next = -1;
    unsigned long long todo = __ballot(unplaced && last >= 0);
    while (todo) {
        int src[4], a[4], be[4];
        bool live[4];
        float ha[4], bh[4];
        const float *h[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            live[k] = todo != 0;                         // wave-uniform
            src[k] = live[k] ? __ffsll(todo) - 1 : src[0];
            if (live[k]) todo &= todo - 1;
            a[k] = __shfl(last, src[k], kWave);
            ha[k] = __shfl(last_h, src[k], kWave);
            h[k] = logits + (size_t)__shfl(tw, src[k], kWave) * E;
            bh[k] = -INFINITY;
            be[k] = 0x7fffffff;
        }
        for (int e = lane; e < E; e += kWave) {
            float v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = h[k][e];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool after = v[k] < ha[k] || (v[k] == ha[k] && e > a[k]);
                if (after && (v[k] > bh[k] || (v[k] == bh[k] && e < be[k]))) { bh[k] = v[k]; be[k] = e; }
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                const float oh = __shfl_xor(bh[k], m, kWave);
                const int oe = __shfl_xor(be[k], m, kWave);
                if (oe != 0x7fffffff && (be[k] == 0x7fffffff || oh > bh[k] || (oh == bh[k] && oe < be[k]))) {
                    bh[k] = oh;
                    be[k] = oe;
                }
            }
            if (live[k] && lane == src[k]) next = be[k] == 0x7fffffff ? -1 : be[k];
        }
    }
    if (unplaced) asked[tw] = next;
}

// -----------------------------------------------------------------------------
// Per 256-token block (never across routing groups): the stage's candidates in token order,
// each one's rank among the block's earlier candidates for the same expert, and the block's
// histogram of experts asked for.
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(kRouteTB) void ntlb_rank_kernel(
    const int32_t *__restrict__ tok_slot, const int32_t *__restrict__ asked,
    int32_t *__restrict__ local_rank, int32_t *__restrict__ block_counts, int nbg, int Tg, int E) {
    extern __shared__ int32_t sm[];
    int32_t *list = sm;                  // [kRouteTB] experts asked for, candidates in token order
    int32_t *wave_n = sm + kRouteTB;     // [4] candidates per wave
    int32_t *hist = sm + kRouteTB + 4;   // [E]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    int t0, tend;
    block_token_range(b, nbg, Tg, t0, tend);
    for (int i = tid; i < E; i += kRouteTB) hist[i] = 0;
    const int tw = t0 + tid;
    const int next = (tw < tend && tok_slot[tw] < 0) ? asked[tw] : -1;
    // position in the block's list = candidates in earlier waves + in earlier lanes;
    // rank = earlier list entries asking for the same expert
    const unsigned long long cmask = __ballot(next >= 0);
    if (lane == 0) wave_n[wave] = __popcll(cmask);
    __syncthreads();
    int before = 0;
    for (int q = 0; q < wave; ++q) before += wave_n[q];
    const int mine = before + __popcll(cmask & ((1ull << lane) - 1ull));
    if (next >= 0) list[mine] = next;
    __syncthreads();
    if (next >= 0) {
        int r = 0;
        for (int q = 0; q < mine; ++q) r += list[q] == next ? 1 : 0;
        local_rank[(size_t)b * kRouteTB + tid] = r;
        atomicAdd(&hist[next], 1);   // integer: order-free
    }
    __syncthreads();
    for (int i = tid; i < E; i += kRouteTB) block_counts[(size_t)b * E + i] = hist[i];
}

// One wave per (group, expert) pair: block_off[b][e] = candidates of e in the group's earlier
// blocks; cnt[g][e] = candidates in the whole group.
__global__ __launch_bounds__(256) void ntlb_block_scan_kernel(
    const int32_t *__restrict__ block_counts, int32_t *__restrict__ block_off,
    int32_t *__restrict__ cnt, int n, int nbg, int E) {
    const int lane = threadIdx.x & 63;
    const long pair = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= (long)n * E) return;
    const int g = (int)(pair / E), e = (int)(pair - (long)g * E);
    int run = 0;
    for (int base = 0; base < nbg; base += kWave) {
        const int bl = base + lane;
        const int c = bl < nbg ? block_counts[((size_t)g * nbg + bl) * E + e] : 0;
        int incl = c;   // inclusive prefix over the lanes
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) {
            const int o = __shfl_up(incl, m, kWave);
            if (lane >= m) incl += o;
        }
        if (bl < nbg) block_off[((size_t)g * nbg + bl) * E + e] = run + incl - c;
        run += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) cnt[pair] = run;
}

// One thread per expert, groups in order.
__global__ __launch_bounds__(256) void ntlb_expert_scan_kernel(
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ counts_g,
    int32_t *__restrict__ used_g, int32_t *__restrict__ kept, int32_t *__restrict__ free_r,
    int32_t *__restrict__ base_r, int n, int E, int C, int Cg, int round) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= E) return;
    const int before = kept[e];   // slots of the expert handed out so far, all groups
    int placed = 0;
    for (int g = 0; g < n; ++g) {
        const size_t pair = (size_t)g * E + e;
        int used;
        if (round == 0) {
            const int c = counts_g[pair];
            used = c < Cg ? c : Cg;
        } else {
            used = used_g[pair];
        }
        const int fr = Cg - used;
        const int want = cnt[pair];
        const int k = want < fr ? want : fr;
        free_r[pair] = fr;
        base_r[pair] = e * C + before + placed;
        used_g[pair] = used + k;
        placed += k;
    }
    kept[e] = before + placed;
}

__global__ __launch_bounds__(256) void ntlb_place_kernel(
    const int32_t *__restrict__ asked, const int32_t *__restrict__ local_rank,
    const int32_t *__restrict__ block_off, const int32_t *__restrict__ free_r,
    const int32_t *__restrict__ base_r, const float *__restrict__ probs,
    int32_t *__restrict__ tok_slot, int32_t *__restrict__ slot_token,
    float *__restrict__ slot_gate, uint32_t *__restrict__ slot_off, uint32_t row_bytes,
    int32_t *__restrict__ idx_ws, float *__restrict__ gate_ws, int32_t *__restrict__ expert_index, float *__restrict__ gate,
    int32_t *__restrict__ pos_out, uint8_t *__restrict__ dropped_out, int T, int Tg, int nbg, int E,
    int Cg) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T || tok_slot[t] >= 0) return;
    const int e = asked[t];
    if (e < 0) return;
    const int g = t / Tg;
    const int b = block_of_token(t, nbg, Tg);
    const int tl = t - (g * Tg + (b - g * nbg) * kRouteTB);
    const int p = block_off[(size_t)b * E + e] + local_rank[(size_t)b * kRouteTB + tl];
    const size_t pair = (size_t)g * E + e;
    const int fr = free_r[pair];
    if (p >= fr) return;   // the expert's capacity ran out before this token's turn
    const int slot = base_r[pair] + p;
    const float pr = probs[(size_t)t * E + e];
    tok_slot[t] = slot;
    slot_token[slot] = t;
    slot_gate[slot] = pr;
    slot_off[slot] = (uint32_t)t * row_bytes;
    idx_ws[t] = e;
    gate_ws[t] = pr;
    expert_index[t] = e;
    gate[t] = pr;
    pos_out[t] = Cg - fr + p;
    dropped_out[t] = 0;
}

hipError_t launch_ntlb(const Workspace &w, char *ws, const float *logits, int32_t *expert_index,
                       float *gate, int32_t *position_in_expert, uint8_t *dropped,
                       hipStream_t s) {
    ProfScope ps("ntlb_stages", s);
    const size_t smem = sizeof(int32_t) * (kRouteTB + 4 + (size_t)w.E);
    for (int round = 0; round < w.ntlb_rounds; ++round) {
        const int W = (int)ceil_div(w.T, kWave);   // waves of the choice kernel
        hipLaunchKernelGGL(ntlb_choice_kernel, dim3((unsigned)ceil_div(W, 4)), dim3(256), 0, s, logits,
                           (const int32_t *)(ws + w.tok_slot), (const int32_t *)(ws + w.idx),
                           (int32_t *)(ws + w.ntlb_asked), (int)w.T, (int)w.E, W, round);
        hipLaunchKernelGGL(ntlb_rank_kernel, dim3((unsigned)w.nb), dim3(kRouteTB), smem, s,
                           (const int32_t *)(ws + w.tok_slot), (const int32_t *)(ws + w.ntlb_asked),
                           (int32_t *)(ws + w.local_rank), (int32_t *)(ws + w.block_counts),
                           (int)w.nbg, (int)w.Tg, (int)w.E);
        hipLaunchKernelGGL(ntlb_block_scan_kernel, dim3((unsigned)ceil_div(w.n * w.E, 4)), dim3(256),
                           0, s, (const int32_t *)(ws + w.block_counts),
                           (int32_t *)(ws + w.block_off), (int32_t *)(ws + w.ntlb_cnt), (int)w.n,
                           (int)w.nbg, (int)w.E);
        hipLaunchKernelGGL(ntlb_expert_scan_kernel, dim3((unsigned)ceil_div(w.E, 256)), dim3(256), 0,
                           s, (const int32_t *)(ws + w.ntlb_cnt), (const int32_t *)(ws + w.counts_g),
                           (int32_t *)(ws + w.ntlb_used), (int32_t *)(ws + w.kept),
                           (int32_t *)(ws + w.ntlb_free), (int32_t *)(ws + w.ntlb_base), (int)w.n,
                           (int)w.E, (int)w.C, (int)w.Cg, round);
        hipLaunchKernelGGL(ntlb_place_kernel, dim3((unsigned)ceil_div(w.T, 256)), dim3(256), 0, s,
                           (const int32_t *)(ws + w.ntlb_asked), (const int32_t *)(ws + w.local_rank),
                           (const int32_t *)(ws + w.block_off), (const int32_t *)(ws + w.ntlb_free),
                           (const int32_t *)(ws + w.ntlb_base), (const float *)(ws + w.probs),
                           (int32_t *)(ws + w.tok_slot), (int32_t *)(ws + w.slot_token),
                           (float *)(ws + w.slot_gate), (uint32_t *)(ws + w.slot_off),
                           (uint32_t)(w.d * w.elt), (int32_t *)(ws + w.idx),
                           (float *)(ws + w.gate), expert_index, gate,
                           position_in_expert, dropped, (int)w.T, (int)w.Tg, (int)w.nbg, (int)w.E,
                           (int)w.Cg);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

}  // namespace sw
