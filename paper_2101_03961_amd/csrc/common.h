// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "switchffn.h"

namespace sw {

typedef __bf16 bf16;

// ---- element helpers -------------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE

constexpr int kWave = 64;

// Entry of the slot -> row-offset table for a slot without a token: as a buffer offset it lies
// beyond every descriptor (all are kept below 2 GB), so loads through it read zeros.
constexpr uint32_t kNoRow = 0x80000000u;

// Token block of the router / position kernels: one block of kRouteTB threads
// owns kRouteTB consecutive tokens.
constexpr int kRouteTB = 256;

// Output tile of the bf16 grouped GEMM (square), and the bytes of ReLU-mask bits per tile.
constexpr int kGemmTile = 256;
constexpr int kReluBitsPerTile = kGemmTile * kGemmTile / 8;

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Token blocks of the router kernels: group g's Tg tokens are cut into nbg blocks of kRouteTB
// (the last one short), so that a block never holds tokens of two routing groups.
__device__ __forceinline__ void block_token_range(int b, int nbg, int Tg, int &t0, int &tend) {
    const int g = b / nbg;
    t0 = g * Tg + (b - g * nbg) * kRouteTB;
    const int gend = (g + 1) * Tg;
    tend = t0 + kRouteTB < gend ? t0 + kRouteTB : gend;
}
__device__ __forceinline__ int block_of_token(int t, int nbg, int Tg) {
    const int g = t / Tg;
    return g * nbg + (t - g * Tg) / kRouteTB;
}
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- training-time noise (Sec. 2.4 expert dropout; App. C input jitter) ------
// Every draw is a function of (seed, stream, element index) only -- 32 bits from
// multiply / xor-shift rounds, documented in switchffn.h -- so any kernel can
// reproduce the draw of an element from its coordinates.
struct Noise {
    uint32_t seed_lo;
    uint32_t jitter_term;    // seed_hi + stream constant of the jitter stream
    uint32_t dropout_term;   // seed_hi + stream constant of the dropout stream
    uint32_t drop_thr;       // a hidden unit is dropped iff its 16 bits are < drop_thr = floor(rate 2^16)
    float drop_scale;        // 2^16 / (2^16 - drop_thr); 1 when dropout is off
    float jitter_eps;
    int dropout, jitter;     // on / off
};
__device__ __forceinline__ uint32_t noise_bits(uint32_t idx, uint32_t seed_lo, uint32_t term) {
    uint32_t z = (idx ^ seed_lo) * 0x9E3779B1u;
    z ^= z >> 15;
    z = (z + term) * 0x85EBCA77u;
    z ^= z >> 13;
    z *= 0xC2B2AE3Du;
    return z ^ (z >> 16);
}
// multiplier of element idx = t * d + k of the router's input: uniform in [1 - eps, 1 + eps)
__device__ __forceinline__ float jitter_of(const Noise &nz, uint32_t idx) {
    const float u = (float)(noise_bits(idx, nz.seed_lo, nz.jitter_term) >> 8) * 0x1p-24f;
    return fmaf(2.0f * nz.jitter_eps, u, 1.0f - nz.jitter_eps);
}
// Expert dropout: the 32 bits drawn for pair i (hidden units 2 i and 2 i + 1 of the flattened
// [token][unit] index) decide both, 16 bits each
__device__ __forceinline__ uint32_t dropout_pair_bits(const Noise &nz, uint32_t pair) {
    return noise_bits(pair, nz.seed_lo, nz.dropout_term);
}
__device__ __forceinline__ bool dropout_keeps_even(const Noise &nz, uint32_t z) {
    return (z & 0xFFFFu) >= nz.drop_thr;
}
__device__ __forceinline__ bool dropout_keeps_odd(const Noise &nz, uint32_t z) {
    return (z >> 16) >= nz.drop_thr;
}
// hidden unit idx = t * f + j survives expert dropout
__device__ __forceinline__ bool dropout_keeps(const Noise &nz, uint32_t idx) {
    const uint32_t z = dropout_pair_bits(nz, idx >> 1);
    return (idx & 1u) ? dropout_keeps_odd(nz, z) : dropout_keeps_even(nz, z);
}

// ---- workspace layout (byte offsets into the caller's workspace) ------------
struct Workspace {
    int64_t T, d, f, E;
    int64_t f1;                 // columns of W_in: f (ReLU FFN) or 2 f (gated-GELU FFN: gate | linear)
    int geglu;                  // gated-GELU FFN
    int64_t n;                  // routing groups
    int64_t Tg;                 // tokens per group (T / n)
    int64_t Cg;                 // capacity: slots per expert and group (Eq. 3 on Tg tokens)
    int64_t C;                  // slots per expert in the expert-major buffers: n * Cg
    int64_t nbg, nb;            // token blocks per group (blocks never straddle groups), in all
    size_t elt;                 // bytes per activation element
    size_t probs;               // f32 [T][E]   router probabilities (saved for backward)
    size_t idx;                 // i32 [T]
    size_t gate;                // f32 [T]
    size_t local_rank;          // i32 [T]      rank among same-expert tokens of the block
    size_t block_counts;        // i32 [nb][E]
    size_t block_psum;          // f32 [nb][E]
    size_t block_off;           // i32 [nb][E]  exclusive prefix of block_counts over blocks
    size_t counts;              // i32 [E]      arg max decisions per expert, all groups
    size_t counts_g;            // i32 [n][E]   ... per group
    size_t psum_g;              // f32 [n][E]   sum of router probabilities per group and expert
    size_t loss_part;           // f64 [8]      parts of sum (counts / Tg) (psum / Tg), one per scan block
    size_t grp_off;             // i32 [n][E]   first slot of group g inside expert e's slots:
                                //              sum of min(counts_g, Cg) over earlier groups
    size_t kept;                // i32 [E]      kept tokens per expert: sum over groups of min(count, Cg)
    int fused;                  // bf16: dispatch and combine run inside the GEMMs (x, dy gathered by
                                //   the slot -> token table, y written by the second GEMM)
    size_t slot_token;          // i32 [E][C] + 128  token held by each slot (valid for slot < kept[e])
    size_t slot_gate;           // f32 [E][C]   gate of that token (the probability that scales its output)
    size_t slot_off;            // u32 [E][C] + 128  byte offset of that token's row in x / dy / y:
                                //              token * d * 2 (only kept when `fused`)
    size_t tok_slot;            // i32 [T]      slot (e * C + grp_off[g][e] + pos) of each kept token,
                                //              -1 for dropped ones
    size_t Xd;                  // act [E][C][d]   dispatched tokens
    size_t H;                   // act [E][C][2f]  Xd W_in = [u | v] (gated-GELU FFN only)
    size_t A;                   // act [E][C][f]   ReLU(Xd W_in), or GELU(u) v; after expert dropout
    size_t O;                   // act [E][C][d]   A W_out
    size_t dO;                  // act [E][C][d]
    size_t dA;                  // act [E][C][f]   dO W_out^T (gated-GELU FFN only)
    size_t dH;                  // act [E][C][f1]  gradient of Xd W_in
    size_t dXd;                 // act [E][C][d]
    size_t dgate;               // f32 [T]
    size_t dlogits;             // f32 [T][E]
    size_t dWr_part;            // f32 [nsplit][d][E]  split-T partial sums of dW_r
    size_t dbr_part;            // f32 [ceil(T / 256)][E]  per-256-token sums of dlogits
    int64_t etiles;             // tiles of 128 experts: ceil(E / 128)
    size_t wsplit;              // bf16 [etiles][3][128][dpad_r]  W_r^T as three bf16 terms (MFMA router)
    int64_t dpad;               // d rounded up to a multiple of 32
    int64_t dpad_r;             // k extent of the MFMA router: dpad, or 3 dpad with input jitter
                                // (the jittered input as three bf16 planes side by side)
    size_t xj;                  // bf16 [T][3 dpad]  x * m as hi | mid | lo planes (jitter + MFMA router)
    size_t no_slot;             // i32 [T]  all -1 (jitter + MFMA router backward)
    size_t wsplit_b;            // bf16 [etiles][d][256]   W_r rows as hi | lo halves (MFMA router backward)
    size_t dl_split;            // bf16 [etiles][T][256]   dlogits rows as hi | lo halves
    size_t dWr_part_m;          // f32 [etiles][nsplit_m][d][256]  partial sums of x^T [dl_hi | dl_lo]
                                //     (with jitter: [nsplit_m][2 dpad][256], hi and mid plane of x * m)
    int64_t tps_m, nsplit_m;    // tokens per split (multiple of 32), number of splits
    size_t relu_bits;           // u8  [E][f tiles][slot tiles][kReluBitsPerTile]  one bit per element of A:
                                //     A > 0, in the order the bf16 GEMM epilogue visits a tile
    int64_t nsplit;
    // No-Token-Left-Behind (only laid out when ntlb_rounds > 0)
    int ntlb_rounds;
    size_t ntlb_logits;         // f32 [T][E]   logits, when the caller asks for none
    size_t ntlb_asked;          // i32 [T]      expert a waiting token asked last (-1: none left)
    size_t ntlb_cnt;            // i32 [n][E]   candidates of the current stage
    size_t ntlb_used;           // i32 [n][E]   slots handed out so far
    size_t ntlb_free;           // i32 [n][E]   capacity free when the current stage starts
    size_t ntlb_base;           // i32 [n][E]   first slot of the current stage's tokens
    size_t total;
    Noise noise;                // not part of the layout: the call's noise parameters
};

int check_config(const switch_config *cfg);
int64_t capacity_of(const switch_config *cfg);
Workspace layout_workspace(const switch_config *cfg);

// ---- one-time set-up per device ------------------------------------------------------
// Kernel attributes (dynamic LDS size) and the CU count belong to a device: each is set or
// read once per device, under std::call_once, by whichever host thread comes first.
constexpr int kMaxDevices = 64;
struct PerDeviceOnce {
    std::once_flag flag[kMaxDevices];
    hipError_t err[kMaxDevices];
};
template <typename F> static inline hipError_t once_per_device(PerDeviceOnce &o, F fn) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return hipErrorInvalidDevice;
    std::call_once(o.flag[dev], [&] { o.err[dev] = fn(); });
    return o.err[dev];
}

// ---- profiling hooks ---------------------------------------------------------
void prof_begin(const char *name, hipStream_t s);
void prof_end(hipStream_t s);

struct ProfScope {
    hipStream_t s;
    ProfScope(const char *name, hipStream_t st) : s(st) { prof_begin(name, st); }
    ~ProfScope() { prof_end(s); }
};

// ---- kernel launchers (each returns hipSuccess or the launch error) ----------
// Router forward: logits, softmax, arg max, gate, in-block rank, per-block
// expert histogram and probability sums.
hipError_t launch_router_fwd(const Workspace &w, int dtype, const void *x, const float *W_r,
                             const float *b_r, char *ws, int32_t *expert_index, float *gate,
                             float *router_logits, hipStream_t s);
// The same on bf16 MFMA (bf16 x, E <= 128, E % 4 == 0): see router_mfma.hip.
bool router_fwd_mfma_supported(const Workspace &w, int dtype);
bool router_bwd_mfma_supported(const Workspace &w, int dtype);
// softmax, arg max, gate, ranks and block statistics from the logits left in the
// probability buffer (the second half of launch_router_fwd)
hipError_t launch_router_softmax(const Workspace &w, char *ws, int32_t *expert_index, float *gate,
                                 float *router_logits, hipStream_t s);
hipError_t launch_router_fwd_mfma(const Workspace &w, const void *x, const float *W_r,
                                  const float *b_r, char *ws, int32_t *expert_index, float *gate,
                                  float *router_logits, hipStream_t s);
// Per-expert scan over token blocks, counts, kept, aux loss.
hipError_t launch_route_scan(const Workspace &w, char *ws, int32_t *expert_counts, hipStream_t s);
// number of blocks of that launch = parts of the loss that positions_kernel adds up
int route_scan_blocks(const Workspace &w);
// Positions, dropped mask, the loss from its parts, gather of kept tokens into expert-major slots.
// With No-Token-Left-Behind stages (logits != nullptr) between the two, which also update
// expert_index and gate of the tokens they place.
hipError_t launch_dispatch(const Workspace &w, int dtype, float alpha, const void *x, char *ws,
                           int32_t *position_in_expert, uint8_t *dropped, float *aux_loss,
                           const float *logits, int32_t *expert_index, float *gate, void *y,
                           hipStream_t s);
hipError_t launch_ntlb(const Workspace &w, char *ws, const float *logits, int32_t *expert_index,
                       float *gate, int32_t *position_in_expert, uint8_t *dropped,
                       hipStream_t s);
// Gated-GELU FFN: A = GELU(u) v (and expert dropout) from H = [u | v]; dH = [du | dv] from dA, H.
hipError_t launch_geglu_fwd(const Workspace &w, int dtype, char *ws, hipStream_t s);
hipError_t launch_geglu_bwd(const Workspace &w, int dtype, char *ws, hipStream_t s);
hipError_t launch_combine(const Workspace &w, int dtype, char *ws, void *y, hipStream_t s);
hipError_t launch_combine_bwd(const Workspace &w, int dtype, const void *dy, char *ws,
                              hipStream_t s);
hipError_t launch_router_bwd(const Workspace &w, int dtype, float alpha, float d_aux,
                             const void *x, const float *W_r, char *ws, void *dx, float *dW_r,
                             float *db_r, hipStream_t s);
// MFMA pieces of the router backward (bf16, E <= 128), in gemm_bf16.hip
hipError_t launch_router_dx_mfma(const Workspace &w, char *ws, void *dx, hipStream_t s);
hipError_t launch_router_dWr_mfma(const Workspace &w, const void *x, char *ws, hipStream_t s);

// Grouped GEMMs over experts.  Each computes, for every expert e,
//   C_e[q][p] = sum_k Q_e(q,k) * P_e(p,k)
// where C_e is row-major with p contiguous.
// (f1 = columns of W_in.  With the gated-GELU FFN the first GEMM stores the plain product
// H = Xd W_in and the second-layer data gradient the plain dA = dO W_out^T; the activation
// and its derivative are applied by the kernels of geglu.hip.)
enum GemmKind {
    GEMM_FWD1,   // A  = relu(Xd W_in) | H = Xd W_in  q: slot  p: f1       k: d_model
    GEMM_FWD2,   // O  = A W_out                  q: slot  p: d_model  k: d_ff
    GEMM_DGRAD2, // dH = (dO W_out^T) * [A > 0] | dA = dO W_out^T   q: slot  p: d_ff  k: d_model
    GEMM_DGRAD1, // dXd = dH W_in^T               q: slot  p: d_model  k: f1
    GEMM_WGRAD2, // dW_out = A^T dO               q: d_ff  p: d_model  k: slot (< kept)
    GEMM_WGRAD1  // dW_in = Xd^T dH               q: d_model p: f1     k: slot (< kept)
};
// The caller's token-major tensors, [T][d_model]: what the GEMMs gather from and scatter to
// when dispatch and combine run inside them (Workspace::fused).
struct TokenMajor {
    const void *x;    // layer input
    const void *dy;   // gradient of the output (backward only)
    void *y;          // layer output (forward only)
};
hipError_t launch_gemm_bf16(GemmKind kind, const Workspace &w, char *ws, const void *W_in,
                            const void *W_out, void *dW_in, void *dW_out, const TokenMajor &tm,
                            hipStream_t s);
hipError_t launch_gemm_f32(GemmKind kind, const Workspace &w, char *ws, const void *W_in,
                           const void *W_out, void *dW_in, void *dW_out, const TokenMajor &tm,
                           hipStream_t s);
// Dispatch and combine inside the GEMMs: the rows of y of tokens without a slot are cleared by
// the kernel that assigns the slots (launch_dispatch) -- unless re-routing stages follow it and
// hand some of those tokens a slot after all; then launch_zero_dropped runs behind them.
inline bool zero_rows_with_positions(const Workspace &w) { return w.fused && w.ntlb_rounds == 0; }
// fused path: +0 rows of y for the tokens without a slot; gate gradient from the saved outputs
hipError_t launch_zero_dropped(const Workspace &w, char *ws, void *y, hipStream_t s);
hipError_t launch_gate_grad(const Workspace &w, const void *dy, char *ws, hipStream_t s);

}  // namespace sw
