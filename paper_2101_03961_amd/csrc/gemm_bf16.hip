// Grouped expert GEMMs on bf16 MFMA (gfx950), fp32 accumulation.
//
// For every expert e the kernel computes tiles of
//     C_e[q][p] = sum_k Q_e(q,k) * P_e(p,k)          (C row-major, p contiguous)
// with a 256 (p) x 256 (q) block tile, four wavefronts in a 2 x 2 arrangement,
// each owning a 128 x 128 sub-tile as 4 x 4 MFMA 32x32x16 tiles (256 fp32
// accumulators per lane).  P feeds the MFMA "A" side, Q the "B" side.
//
// Data path.  Operand tiles go from HBM/L2 straight into LDS with
// buffer_load_dwordx4 ... lds (no registers, no ds_write: LDS stores issued by
// the waves cost ~30 cycles of issue each and were the bottleneck of an earlier
// register-staged version).  k advances 64 at a time: every row of an operand tile
// is then one full 128-byte line per step.  One operand goes through three LDS stages of
// 32 KB (the "deep" ring), the other through two (3 x 32 + 2 x 32 = all 160 KB).  The deep
// one is P unless DEEP_Q is set; which is better was measured per GEMM (see
// launch_gemm_bf16), the wrong choice costs 4-11 %.  Below, P is the deep one.  In the
// last quarter of step kt, right after the barrier that frees the stages of step
// kt, a wave issues its eight loads of Q for step kt+2 and then its eight loads of P
// for step kt+3.  Loads complete in order, so the wait of step kt+1 (for step kt+2's
// operands) leaves the eight youngest -- P of step kt+3 -- in flight: the weights are
// asked for a whole step earlier than a two-stage ring allows.  (Measured with the
// loads of the first forward GEMM and 64 MFMAs per step and wave, no LDS reads:
// two stages each 352 us, this arrangement 268 us, three stages each 240 us = the
// time of the loads alone.  With one step of lead a CU has one stage of requests
// outstanding and the fetch path, which needs about two to run at its rate, idles.)
//   - An operand stored [row][k] (k contiguous) is kept in LDS as [row][64 k];
//     a lane's MFMA fragment (8 consecutive k of one row) is one ds_read_b128.
//   - An operand stored [k][row] (row contiguous: the weights in the forward
//     pass, both operands of the weight-gradient GEMMs) is kept in LDS exactly
//     as in memory, [64 k][256 rows], and fragments are fetched with the
//     transposing LDS read ds_read_b64_tr_b16 (two per fragment), which hands
//     each lane four consecutive k of its own row.
//   In both layouts the 16-byte chunks of an LDS row are XOR-permuted (the
//   permutation is applied to the global address each lane fetches, since the
//   LDS side of a direct load is fixed to lane * 16) so that fragment reads
//   spread over all banks.
//
// Schedule per k step and wave: 64 MFMAs in four sub-steps of 16.  Fragments are
// double buffered in registers and read one sub-step ahead; the single barrier
// of the step sits before the last sub-step, so the MFMA pipe always has that
// sub-step's work queued while waves meet.
//
// Ragged edges cost no branches: loads are bounded by the buffer descriptor
// (rows past the expert's kept tokens, k past the reduction length read as
// zero), and lanes whose chunk is invalid in the other dimension use an offset
// beyond every descriptor.
//
// Work assignment: persistent blocks, one per CU, each walking a strided list of
// (expert, p tile, q tile) tiles of its XCD; q tiles beyond the expert's
// kept-token count are skipped.  Tiles that share an operand tile run at the same
// time on one XCD and walk k in the same order, so that each line is fetched from
// HBM once per XCD (measured: starting neighbours a few k steps apart, to turn
// hits under a miss into plain hits, raised HBM traffic by a third -- the leading
// block's lines were evicted before the followers arrived -- and saved no time).
// The k steps of all tiles of a block form one load pipeline: a tile's last steps issue
// the next tile's first loads, which stay in flight during the epilogue.
// The epilogue turns each wave's sub-tile around, 32 rows at a time, through 8 KB of
// LDS of its own -- a quarter of the deep ring's stage that the tile's last step has freed; the
// load that stage is waiting for (the deep operand of the next tile's third step) is issued after the
// epilogue instead of before it -- so that C is written in whole 256-byte row
// segments; fused into it: ReLU and one mask bit per element
// (first forward GEMM), that mask (gradient w.r.t. the hidden activations), the
// gathered addend of the router's dx.  The expert GEMMs' stores are buffer stores of a
// fixed number per lane (rows and columns that do not exist fall outside the descriptor),
// and nothing waits for them: loads and stores retire in order, so the next tile's first
// step simply counts them among the operations that may stay in flight.  (Measured: the
// k loops alone run 229-267 us per launch at Switch-Base, the epilogue's instructions cost
// 10-45 us, the writes to HBM themselves another 30-60 us whether or not they are waited for.)
//
// Dispatch and combine (Sec. 5.4) without a pass of their own (on request: at the Switch-Base
// shape the gathers below cost a little more than the passes they replace).  With GATHER set an operand's
// rows are fetched from the token-major tensors by the slot -> token table: the first forward
// GEMM and the first-layer weight gradient read x, the second-layer data and weight gradients
// read dy.  The first GEMM's epilogue scales each hidden row by its token's gate (EPI_SCALE) so
// that the second GEMM's rows are the layer's output rows, which its epilogue writes straight
// to y[token] (EPI_SCATTER, next to the slot-major copy the gate gradient reads); the second-
// layer data gradient applies the gate as a row scale likewise, (g dy) W^T = g (dy W^T), and
// the second-layer weight gradient needs no scaled dy at all: (g A)^T dy = A^T (g dy).
#include "common.h"
#include "lds_operands.h"

namespace sw {

constexpr int kBP = kGemmTile;                    // block tile, p rows
constexpr int kBQ = kGemmTile;                    // block tile, q rows
constexpr int kBK = 64;                           // k per pipeline step
constexpr int kDeepStages = 3;                    // LDS stages of the operand that mostly comes from HBM
constexpr int kShallowStages = 2;                 // ... of the other operand
constexpr int kGemmThreads = 256;
static_assert(kOpBytes64 == kBP * kBK * 2, "operand stage size");
constexpr int kDeepRingBytes = kDeepStages * kOpBytes64;      // 96 KB
constexpr int kRingBytes = kDeepRingBytes + kShallowStages * kOpBytes64;   // 160 KB: all of a CU's LDS
constexpr int kTurnBytes = 32 * 256;              // per wave: 32 rows x 128 bf16 of the epilogue's turn-around
static_assert(4 * kTurnBytes == kOpBytes64, "the turn-around buffers are one stage of the deep ring");
constexpr int kGemmLds = kRingBytes;
constexpr int kXcds = 8;

struct GemmArgs {
    const bf16 *Q;      // per expert: q_batch elements
    const bf16 *P;
    bf16 *Cout;
    const bf16 *mask;   // ROUTER_DX: rows added to the product in the epilogue
    uint8_t *relu_bits; // EPI_RELU writes, EPI_MASK reads: one bit per output element, tile-private order
    size_t q_batch, p_batch, c_batch;
    int ldq, ldp, ldc;  // leading dimensions in elements
    int Qdim, Pdim, Kdim;
    const int32_t *kept;
    int tiles_q, tiles_p, total_tiles;
    int reverse;        // walk the experts from the last to the first (see launch_gemm_bf16)
    // router backward uses of the kernel (see GemmMode)
    const int32_t *slot_token;          // EPI_DROP: token of each slot, [expert][slots]
    int slots;                          //           slots per expert
    Noise nz;                           //           dropout threshold, scale, seed
    const int32_t *tok_slot;            // ROUTER_DX: row of the addend for each token, -1: none
    int router_tiles;                   // ROUTER_DX: tiles of 128 experts; operands are planes
    int q_plane, p_plane;               //   [tile][row][256], plane sizes in elements
    float *Cf;                          // ROUTER_DWR: fp32 partial sums [split][q][p]
    int T_total, tps;                   // ROUTER_DWR: tokens, tokens per split
    // dispatch / combine inside the GEMM (see GATHER, EPI_SCALE, EPI_SCATTER)
    uint32_t gather_bytes;              // bytes of a token-major matrix (gathered operand, Cscatter)
    const uint32_t *slot_off;           // byte offset of each slot's token row in the token-major tensors
    const float *row_scale;             // EPI_SCALE: gate of each slot's token, [expert][slots]
    bf16 *Cscatter;                     // EPI_SCATTER: token-major output, row token(slot)
};

// What the "experts" and the k dimension of a launch are.
//   EXPERTS     the grouped expert GEMMs: batch = experts, limits from kept[].
//   ROUTER_DX   dx = dl W_r^T + gathered dXd: one batch; k runs over three blocks of
//               128 experts pairing the bf16 halves of dl (hi|lo per row, 256 wide)
//               with those of W_r^T (hi|lo per row): hi*hi, hi*lo, lo*hi.
//   ROUTER_DWR  partial sums of x^T [dl_hi | dl_lo] over token ranges: batch = token
//               range, k = tokens of the range, fp32 output.
enum GemmMode { MODE_EXPERTS = 0, MODE_ROUTER_DX = 1, MODE_ROUTER_DWR = 2 };

template <bool TRANS, bool GATHER> struct OperandOf { typedef DirectOperand64 type; };
template <> struct OperandOf<true, false> { typedef TransOperand64 type; };
template <> struct OperandOf<false, true> { typedef DirectGather64 type; };
template <> struct OperandOf<true, true> { typedef TransGather64 type; };
// which operands are gathered by the slot -> token table
enum { GATHER_NONE = 0, GATHER_Q = 1, GATHER_P = 2 };

// EPI_DROP is a flag on top of EPI_RELU / EPI_MASK: expert dropout (Sec. 2.4) zeroes hidden
// units after the ReLU and scales the survivors; the mask bits then say "active and kept",
// and the masked gradient is scaled by the same factor.
// EPI_SCALE multiplies every output row by its slot's gate before the store (after ReLU and
// dropout; the mask bits are taken from the stored values, and gate > 0).  EPI_SCATTER also
// writes every output row to row token(slot) of a token-major tensor.
enum { EPI_NONE = 0, EPI_RELU = 1, EPI_MASK = 2, EPI_DROP = 4, EPI_SCALE = 8, EPI_SCATTER = 16 };

// One output tile of one expert.
struct Tile {
    int e, p0, q0, qlim, klim;
    int index;      // number of the tile among all tiles of the launch
};

// Tiles are numbered expert-major; inside an expert the dimension with fewer tiles runs
// fastest, so that the tiles sharing a tile of the larger operand are neighbours.  The
// number line is cut into kXcds equal ranges, one per XCD.  Block b runs on XCD
// b % kXcds (workgroups are dealt to XCDs round-robin) and walks that XCD's range
// with the stride of the blocks sharing the XCD, so at any moment the CUs of an
// XCD work on neighbouring tiles -- the q tiles that share a weight tile, the p
// tiles that share an activation tile -- and find each other's data in their L2.
template <bool Q_LIMITED, bool K_LIMITED, int MODE>
__device__ __forceinline__ bool next_tile(const GemmArgs &a, int &L, int L_end, int stride,
                                          Tile &t) {
    const int tiles_pe = a.tiles_q * a.tiles_p;
    for (; L < L_end; L += stride) {
        const int e_fwd = L / tiles_pe;
        const int rem = L - e_fwd * tiles_pe;
        const int e = a.reverse ? a.total_tiles / tiles_pe - 1 - e_fwd : e_fwd;
        int pt, qt;
        if (a.tiles_q <= a.tiles_p) {
            pt = rem / a.tiles_q;
            qt = rem - pt * a.tiles_q;
        } else {
            qt = rem / a.tiles_p;
            pt = rem - qt * a.tiles_p;
        }
        int kept = 0;
        if (MODE == MODE_EXPERTS) kept = a.kept[e];
        if (MODE == MODE_ROUTER_DWR) kept = min(a.tps, a.T_total - e * a.tps);
        t.e = e;
        t.p0 = pt * kBP;
        t.q0 = qt * kBQ;
        t.index = e * tiles_pe + rem;
        t.qlim = Q_LIMITED ? (kept < a.Qdim ? kept : a.Qdim) : a.Qdim;
        t.klim = K_LIMITED ? (kept < a.Kdim ? kept : a.Kdim) : a.Kdim;
        if (t.q0 < t.qlim) {   // q tiles past the expert's kept tokens have no work
            L += stride;
            return true;
        }
    }
    return false;
}

// wait until at most N of this wave's direct loads and stores are still in flight
#define SW_WAIT_VMCNT(N) asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory")
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "the counter has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// One store of 16 bytes per lane at byte offset voff of the buffer; offsets past the buffer's
// size store nothing.  Written as asm so that every lane's store is issued whatever its
// offset -- the number of stores in flight is then known -- and so that the compiler's own
// waits do not count it.  The compiler does not look into asm for hazards: the leading s_nop
// keeps five states between a descriptor word it may just have reloaded from a spill lane
// (v_readlane) and the store that reads it, the trailing one keeps a write of the data
// registers one state away.
__device__ __forceinline__ void store16(i32x4 rsrc, uint32_t voff, u32x4 data) {
    asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, 0 offen\n\ts_nop 0"
                 :
                 : "v"(data), "v"(voff), "s"(rsrc)
                 : "memory");
}

// two floats rounded to bf16 (nearest even), first in the low half
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
// per 16-bit half: signed maximum, unsigned minimum (written as asm: the compiler turns the
// generic forms of these into compares and selects, several instructions per half)
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_pk_max_i16 %0, %1, %2" : "=v"(d) : "v"(x), "v"(y));
    return d;
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(d) : "v"(x), "v"(y));
    return d;
}

// Per-tile values of the epilogue, one set per lane (see tile_values in the kernel).
struct TileVals {
    uint32_t ep_lo, ep_hi;   // SCALE / SCATTER: gate / row offset of rows lane, lane + 64 of the wave's q rows
    uint32_t mb[8];          // EPI_MASK: the lane's 32 bytes of ReLU bits of the tile
    int slot_lo, slot_hi;    // ROUTER_DX: slot of the addend of rows lane, lane + 64 (-1: none)
    int tok_lo, tok_hi;      // EPI_DROP after ReLU: token of those rows
};

template <bool Q_TRANS, bool P_TRANS, int EPI, bool Q_LIMITED, bool K_LIMITED, int MODE, int GATHER,
          bool DEEP_Q>
__global__ __launch_bounds__(kGemmThreads) void gemm_bf16_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int EPI_BASE = EPI & 3;
    constexpr bool DROP = (EPI & EPI_DROP) != 0;
    constexpr bool SCALE = (EPI & EPI_SCALE) != 0;
    constexpr bool SCATTER = (EPI & EPI_SCATTER) != 0;
    constexpr bool GQ = (GATHER & GATHER_Q) != 0, GP = (GATHER & GATHER_P) != 0;
    constexpr bool GQ_ROWS = GQ && !Q_TRANS;            // Q's tile rows are gathered (per tile)
    static_assert(!(GP && !P_TRANS), "P is gathered only along k");
    static_assert(!(SCALE && SCATTER), "one per-row table per launch");
    // The bf16 epilogue of the expert GEMMs issues a fixed number of stores per lane and does
    // not wait for them: the next tile's first step counts them among the operations that may
    // stay in flight, the second waits for loads issued after them and thereby for them.
    constexpr bool ASYNC_STORES = MODE == MODE_EXPERTS;
    constexpr int kEpStores = ASYNC_STORES ? (SCATTER ? 64 : 32) + (EPI_BASE == EPI_RELU ? 2 : 0) : 0;
    constexpr int kFirstWait = 8 + kEpStores > 63 ? 63 : 8 + kEpStores;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave & 1;
    const int wq = wave >> 1;
    // tile row of row r of 32-row block j of wave row w
    auto row_of = [](int w, int j, int r) { return w * 128 + j * 32 + r; };
    // LDS address of the ring (the dynamic segment starts the block's allocation)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;

    // persistent block: one per CU, a strided walk over its XCD's tile range
    const int per_xcd = (a.total_tiles + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds;
    const int stride = gridDim.x / kXcds;
    int L = xcd * per_xcd + blockIdx.x / kXcds;
    const int L_end = min((xcd + 1) * per_xcd, a.total_tiles);

    Tile cur, nxt, after;
    if (!next_tile<Q_LIMITED, K_LIMITED, MODE>(a, L, L_end, stride, cur)) return;

    // The k steps of all tiles of this block form one pipeline: while a tile's last steps are
    // multiplied, the loads of the next tile's first steps are already under way, and they stay
    // in flight during the epilogue.  A tile takes at least three steps (steps past its k range
    // read zeros).  The two operands run through their rings separately: P three steps ahead of
    // the step that issues its loads, Q two, so each has its own "tile the loads are in".
    auto steps_of = [&](const Tile &t) { return (t.klim + kBK - 1) / kBK; };
    typename OperandOf<P_TRANS, GP>::type op;
    typename OperandOf<Q_TRANS, GQ>::type oq;
    op.init_frag(lane, wp * 128);
    oq.init_frag(lane, wq * 128);
    int ldp_nk = 0, ldq_nk = 0;   // k steps (with data) of the tile the P / Q loads are in
    int ldp_e = 0, ldq_e = 0;     // its expert
    // Values fetched with ordinary loads long before their use, and "pinned" (passed through an
    // empty asm) right after a k step's barrier: the wait the compiler puts before their first
    // use counts only the loads it knows of, so it also sits out every direct load issued
    // before them; after a step's own wait that costs little, in front of the epilogue or of
    // the next tile's loads it would cost a fetch latency per tile.
    // (row offsets: byte offset of a slot's token row in the token-major tensors, slot_off)
    uint32_t off_rows = kOobOffset;  // GQ_ROWS: offset of row 8 wave + (lane & 7) + 32 (lane >> 3) of the next tile
    // k-rows gathered: offsets of the wave's sixteen k-rows 16 wave .. of the step to be loaded; they are
    // the same for all lanes of a half wave, so they are fetched by scalar loads, which the
    // counter of the direct loads does not see
    uint32_t off_step[16] = {kOobOffset, kOobOffset, kOobOffset, kOobOffset, kOobOffset, kOobOffset,
                             kOobOffset, kOobOffset, kOobOffset, kOobOffset, kOobOffset, kOobOffset,
                             kOobOffset, kOobOffset, kOobOffset, kOobOffset};
    TileVals tv = {}, tvn = {};      // epilogue values of the current tile, of the next one
    auto rows_offsets = [&](const Tile &t) {
        const int row = t.q0 + 8 * wave + (lane & 7) + 32 * (lane >> 3);
        return row < t.qlim ? a.slot_off[(size_t)t.e * a.slots + row] : kOobOffset;
    };
    auto begin_p = [&](const Tile &t) {
        if (MODE == MODE_ROUTER_DX) {
            // the 384 k values of an expert tile are read from 256-wide (hi | lo) rows of that
            // tile's plane; k offsets address across planes, so the bounds span all of them (a
            // ragged last row tile then reads rows of the next plane: finite, and never stored)
            op.init_load(a.P, a.ldp, t.p0, a.router_tiles * a.Pdim, a.router_tiles * a.p_plane, lane,
                         wave);
        } else if constexpr (GP) {
            op.init_gather(a.P, a.gather_bytes, t.p0, a.Pdim, lane, wave);
        } else {
            op.init_load(a.P + (size_t)t.e * a.p_batch, a.ldp, t.p0, a.Pdim, t.klim, lane, wave);
        }
        ldp_nk = steps_of(t);
        ldp_e = t.e;
    };
    auto begin_q = [&](const Tile &t) {
        if (MODE == MODE_ROUTER_DX) {
            oq.init_load(a.Q, a.ldq, t.q0, a.router_tiles * a.Qdim, a.router_tiles * a.q_plane, lane,
                         wave);
        } else if constexpr (GQ_ROWS) {
            oq.init_gather(a.Q, a.gather_bytes, t.klim, lane, wave, off_rows);
        } else if constexpr (GQ) {
            oq.init_gather(a.Q, a.gather_bytes, t.q0, t.qlim, lane, wave);
        } else {
            oq.init_load(a.Q + (size_t)t.e * a.q_batch, a.ldq, t.q0, t.qlim, t.klim, lane, wave);
        }
        ldq_nk = steps_of(t);
        ldq_e = t.e;
    };
    // row offsets of the k-rows of step r of expert e.  Slots without a token hold kOobOffset,
    // and the table is padded for steps past the end.  (Read through the constant address
    // space: the table was written by an earlier kernel.)
    auto step_offsets = [&](int e, int r) {
        typedef const __attribute__((address_space(4))) uint32_t *const_u32_ptr;
        const_u32_ptr row = (const_u32_ptr)(uintptr_t)(a.slot_off + (size_t)e * a.slots + r * kBK + 16 * wave);
#pragma unroll
        for (int i = 0; i < 16; ++i) off_step[i] = row[i];
    };
    // load i of a lane fetches k-row 16 wave + 2 i + lane / 32
    auto step_offset_of = [&](int i) { return lane < 32 ? off_step[2 * i] : off_step[2 * i + 1]; };
    // k offset of step j of the tile the P (Q) loads are in; steps past its range read zeros
    int k0p_ = 0, k0q_ = 0;
    auto k_of_p = [&](int j) {
        const int r = j < ldp_nk ? j : ldp_nk;
        if (GP) step_offsets(ldp_e, r);
        if (MODE == MODE_ROUTER_DX) {
            // six steps per expert tile -- 0,1: dl_hi x W_hi, 2,3: dl_hi x W_lo, 4,5: dl_lo x W_hi --
            // in that tile's planes; past the last tile: beyond the k limit (zeros)
            const int jt = r / 6, rr = r - 6 * jt;
            k0p_ = jt * a.p_plane + (rr < 2 ? 64 * rr : (rr < 4 ? 128 + 64 * (rr - 2) : 64 * (rr - 4)));
            if (r >= ldp_nk) k0p_ = a.router_tiles * a.p_plane;
        } else {
            k0p_ = r * kBK;
        }
    };
    auto k_of_q = [&](int j) {
        const int r = j < ldq_nk ? j : ldq_nk;
        if (GQ && Q_TRANS) step_offsets(ldq_e, r);
        if (MODE == MODE_ROUTER_DX) {
            const int jt = r / 6, rr = r - 6 * jt;
            k0q_ = jt * a.q_plane + (rr < 4 ? 64 * (rr & 1) : 128 + 64 * (rr - 4));
            if (r >= ldq_nk) k0q_ = a.router_tiles * a.q_plane;
        } else {
            k0q_ = r * kBK;
        }
    };

    auto pin_tile_values = [&](TileVals &v) {
        if (SCALE || SCATTER) asm volatile("" : "+v"(v.ep_lo), "+v"(v.ep_hi));
        if (EPI_BASE == EPI_MASK)
            asm volatile("" : "+v"(v.mb[0]), "+v"(v.mb[1]), "+v"(v.mb[2]), "+v"(v.mb[3]), "+v"(v.mb[4]),
                              "+v"(v.mb[5]), "+v"(v.mb[6]), "+v"(v.mb[7]));
        if (MODE == MODE_ROUTER_DX) asm volatile("" : "+v"(v.slot_lo), "+v"(v.slot_hi));
        if (DROP && EPI_BASE == EPI_RELU) asm volatile("" : "+v"(v.tok_lo), "+v"(v.tok_hi));
    };
    auto pin_values = [&]() {
        if (GQ_ROWS) asm volatile("" : "+v"(off_rows));
        pin_tile_values(tv);
        pin_tile_values(tvn);
    };

    // fragments: two register sets, each fragment as two 8-byte halves
    s16x4 fa[2][4][2], fb[2][4][2];
    constexpr int kNP = OperandOf<P_TRANS, GP>::type::kPieces;
    constexpr int kNR = kNP + OperandOf<Q_TRANS, GQ>::type::kPieces;   // LDS reads per sub-step

// The two rings: the deep one (three stages, the first 96 KB) carries the operand that mostly
// comes from HBM -- P, or with DEEP_Q Q (the second-layer weight gradient, whose Q is the
// hidden activations and whose P is dy) -- the shallow one (two stages) the other.
// Byte offsets of stage DST of the deep ring, SST of the shallow ring, of the stages that hold P / Q:
#define SW_DEEP_AT(DST) ((DST) * kOpBytes64)
#define SW_SHALLOW_AT(SST) (kDeepRingBytes + (SST) * kOpBytes64)
#define SW_P_AT(DST, SST) (DEEP_Q ? SW_SHALLOW_AT(SST) : SW_DEEP_AT(DST))
#define SW_Q_AT(DST, SST) (DEEP_Q ? SW_DEEP_AT(DST) : SW_SHALLOW_AT(SST))
// direct load G of eight of the P (Q) operand into the stage at byte offset AT
#define SW_ISSUE_P_AT(AT, G)                                                          \
    do {                                                                              \
        const uint32_t st_ = lds0 + (uint32_t)(AT);                                   \
        if constexpr (GP) op.issue_one(st_, wave, (G), step_offset_of(G));            \
        else op.issue_one(st_, k0p_, wave, (G));                                      \
    } while (0)
#define SW_ISSUE_Q_AT(AT, G)                                                          \
    do {                                                                              \
        const uint32_t st_ = lds0 + (uint32_t)(AT);                                   \
        if constexpr (GQ && Q_TRANS) oq.issue_one(st_, wave, (G), step_offset_of(G)); \
        else oq.issue_one(st_, k0q_, wave, (G));                                      \
    } while (0)
// ... of the deep (shallow) operand into stage DST (SST) of its ring
#define SW_ISSUE_DEEP(DST, G)                                                         \
    do {                                                                              \
        if constexpr (DEEP_Q) SW_ISSUE_Q_AT(SW_DEEP_AT(DST), G);                      \
        else SW_ISSUE_P_AT(SW_DEEP_AT(DST), G);                                       \
    } while (0)
#define SW_ISSUE_SHALLOW(SST, G)                                                      \
    do {                                                                              \
        if constexpr (DEEP_Q) SW_ISSUE_P_AT(SW_SHALLOW_AT(SST), G);                   \
        else SW_ISSUE_Q_AT(SW_SHALLOW_AT(SST), G);                                    \
    } while (0)
// LDS reads [G kNR/8, (G+1) kNR/8) of the fragments of the step in stages DST / SST, sub-step KS into SET
#define SW_READ_GROUP(SET, DST, SST, KS, G)                                           \
    do {                                                                              \
        const char *sp_ = lds + SW_P_AT(DST, SST);                                    \
        const char *sq_ = lds + SW_Q_AT(DST, SST);                                    \
        _Pragma("unroll") for (int x_ = (G)*kNR / 8; x_ < ((G) + 1) * kNR / 8; ++x_) { \
            if (x_ < kNP) op.read_piece(sp_, x_, KS, fa[SET]);                        \
            else oq.read_piece(sq_, x_ - kNP, KS, fb[SET]);                           \
        }                                                                             \
    } while (0)
// MFMAs 2 G and 2 G + 1 of the sixteen of a sub-step (fragment pairs in row-major order)
#define SW_MFMA_PAIR(SET, G)                                                          \
    _Pragma("unroll") for (int m_ = 2 * (G); m_ < 2 * (G) + 2; ++m_) {                \
        const int i_ = m_ >> 2, j_ = m_ & 3;                                          \
        const s16x8 a8_ = __builtin_shufflevector(fa[SET][i_][0], fa[SET][i_][1], 0, 1, 2, 3, 4, 5, 6, 7); \
        const s16x8 b8_ = __builtin_shufflevector(fb[SET][j_][0], fb[SET][j_][1], 0, 1, 2, 3, 4, 5, 6, 7); \
        acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                        \
            __builtin_bit_cast(bf16x8, a8_), __builtin_bit_cast(bf16x8, b8_), acc[i_][j_], 0, 0, 0); \
    }

// One k step = four sub-steps of 16 MFMAs, on the operands in deep stage dst and shallow stage
// sst.  Fragments of a sub-step are read (into the other of two register sets) between the MFMAs
// of the sub-step before it.  After the third sub-step's MFMAs nobody reads these stages any
// more: the step's one barrier sits there, behind a wait that leaves the eight youngest loads
// (the deep operand of the step after next) in flight.  The fourth sub-step runs with the loads
// of the shallow operand for the step after next (into the shallow stage just freed), then --
// unless ISSUE_DEEP is false -- of the deep operand for the step after that (into the deep stage
// just freed; k offsets from the preceding k_of_shallow / k_of_deep), and with the first
// fragments of the next step between its MFMAs.
#define SW_K_STEP(ISSUE_DEEP)                                                         \
    do {                                                                              \
        const int dn_ = dst == kDeepStages - 1 ? 0 : dst + 1;                         \
        _Pragma("unroll") for (int g = 0; g < 8; ++g) {                               \
            SW_READ_GROUP(1, dst, sst, 1, g);                                         \
            SW_MFMA_PAIR(0, g)                                                        \
            __builtin_amdgcn_sched_barrier(0);                                        \
        }                                                                             \
        _Pragma("unroll") for (int g = 0; g < 8; ++g) {                               \
            SW_READ_GROUP(0, dst, sst, 2, g);                                         \
            SW_MFMA_PAIR(1, g)                                                        \
            __builtin_amdgcn_sched_barrier(0);                                        \
        }                                                                             \
        _Pragma("unroll") for (int g = 0; g < 8; ++g) {                               \
            SW_READ_GROUP(1, dst, sst, 3, g);                                         \
            SW_MFMA_PAIR(0, g)                                                        \
            __builtin_amdgcn_sched_barrier(0);                                        \
        }                                                                             \
        if (first_step) { /* after an epilogue: its stores and the deep operand of step 2 are younger */ \
            wait_vmcnt<kFirstWait>();                                                 \
            first_step = false;                                                       \
        } else {                                                                      \
            SW_WAIT_VMCNT(8); /* the next step has landed */                          \
        }                                                                             \
        __syncthreads();                                                              \
        pin_values();                                                                 \
        _Pragma("unroll") for (int g = 0; g < 8; ++g) {                               \
            if (g < 4) {                                                              \
                SW_ISSUE_SHALLOW(sst, 2 * g);                                         \
                SW_ISSUE_SHALLOW(sst, 2 * g + 1);                                     \
            } else if (ISSUE_DEEP) {                                                  \
                SW_ISSUE_DEEP(dst, 2 * (g - 4));                                      \
                SW_ISSUE_DEEP(dst, 2 * (g - 4) + 1);                                  \
            }                                                                         \
            SW_READ_GROUP(0, dn_, sst ^ 1, 0, g);                                     \
            SW_MFMA_PAIR(1, g)                                                        \
            __builtin_amdgcn_sched_barrier(0);                                        \
        }                                                                             \
        dst = dn_;                                                                    \
        sst ^= 1;                                                                     \
    } while (0)

    // the operand in the deep ring and the one in the shallow ring
    auto begin_deep = [&](const Tile &t) { if constexpr (DEEP_Q) begin_q(t); else begin_p(t); };
    auto begin_shallow = [&](const Tile &t) { if constexpr (DEEP_Q) begin_p(t); else begin_q(t); };
    auto k_of_deep = [&](int j) { if constexpr (DEEP_Q) k_of_q(j); else k_of_p(j); };
    auto k_of_shallow = [&](int j) { if constexpr (DEEP_Q) k_of_p(j); else k_of_q(j); };
    auto disable_deep = [&]() { if constexpr (DEEP_Q) oq.disable_load(); else op.disable_load(); };
    auto disable_shallow = [&]() { if constexpr (DEEP_Q) op.disable_load(); else oq.disable_load(); };

    int dst = 0, sst = 0;   // stages of the step that is multiplied next
    bool first_step = false;   // the step that is multiplied next follows an epilogue
    // per-tile values of the epilogue, asked for two steps before the end of the tile before
    // (see pin_values)
    auto tile_values = [&](const Tile &t, TileVals &v) {
        if (MODE == MODE_ROUTER_DX) {
            // slot of the addend of rows lane and lane + 64 of the wave's 128 rows
            // (-1: dropped token or past the end: nothing to add)
            const int q = t.q0 + wq * 128 + lane;
            v.slot_lo = q < t.qlim ? a.tok_slot[q] : -1;
            v.slot_hi = q + 64 < t.qlim ? a.tok_slot[q + 64] : -1;
        }
        if (EPI_BASE == EPI_MASK) {
            const uint32_t *bits = (const uint32_t *)(a.relu_bits + (size_t)t.index * kReluBitsPerTile +
                                                      (size_t)(wave * 64 + lane) * 32);
            const u32x4 b0 = *(const u32x4 *)bits, b1 = *(const u32x4 *)(bits + 4);
#pragma unroll
            for (int w = 0; w < 4; ++w) { v.mb[w] = b0[w]; v.mb[4 + w] = b1[w]; }
        }
        if (SCALE || SCATTER || (DROP && EPI_BASE == EPI_RELU)) {
            // gate (SCALE) or row offset (SCATTER) of the wave's q rows: lane 32 j + r holds the
            // value of row r of the wave's block j (ep_lo: j = 0, 1; ep_hi: j = 2, 3)
            const int q_lo = t.q0 + row_of(wq, lane >> 5, lane & 31);
            const int q_hi = t.q0 + row_of(wq, 2 + (lane >> 5), lane & 31);
            const size_t at = (size_t)t.e * a.slots;
            if (SCALE) {
                v.ep_lo = q_lo < t.qlim ? __float_as_uint(a.row_scale[at + q_lo]) : 0u;
                v.ep_hi = q_hi < t.qlim ? __float_as_uint(a.row_scale[at + q_hi]) : 0u;
            }
            if (SCATTER) {   // rows without a token: an offset past the output
                v.ep_lo = q_lo < t.qlim ? a.slot_off[at + q_lo] : kOobOffset;
                v.ep_hi = q_hi < t.qlim ? a.slot_off[at + q_hi] : kOobOffset;
            }
            if (DROP && EPI_BASE == EPI_RELU) {
                v.tok_lo = q_lo < t.qlim ? a.slot_token[at + q_lo] : 0;
                v.tok_hi = q_hi < t.qlim ? a.slot_token[at + q_hi] : 0;
            }
        }
    };

    // Start of the pipeline: both operands of the first tile's steps 0 and 1, then the deep one
    // of step 2; step 0 is awaited (what may stay in flight: both of step 1 and the deep one of
    // step 2, 24 loads).
    tile_values(cur, tv);
    if (GQ_ROWS) off_rows = rows_offsets(cur);
    begin_p(cur);
    begin_q(cur);
    bool have_next = next_tile<Q_LIMITED, K_LIMITED, MODE>(a, L, L_end, stride, nxt);
    // rows of the tile after (pinned after a barrier, used when its loads begin)
    if (GQ_ROWS && have_next) off_rows = rows_offsets(nxt);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        k_of_shallow(st);
#pragma unroll
        for (int g = 0; g < 8; ++g) SW_ISSUE_SHALLOW(st, g);
        k_of_deep(st);
#pragma unroll
        for (int g = 0; g < 8; ++g) SW_ISSUE_DEEP(st, g);
    }
    k_of_deep(2);
#pragma unroll
    for (int g = 0; g < 8; ++g) SW_ISSUE_DEEP(2, g);
    SW_WAIT_VMCNT(24);
    __syncthreads();

    while (true) {
        const int nsteps = steps_of(cur) > 3 ? steps_of(cur) : 3;
        auto bits_of = [&](int ln) {
            return (uint32_t *)(a.relu_bits + (size_t)cur.index * kReluBitsPerTile +
                                (size_t)(wave * 64 + ln) * 32);
        };

        f32x16 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // first fragments of the tile's first step (it has landed: awaited in the step before)
#pragma unroll
        for (int g = 0; g < 8; ++g) SW_READ_GROUP(0, dst, sst, 0, g);

        // Step kt issues the shallow operand of step kt + 2 and the deep one of step kt + 3 of
        // this tile, as long as there are such steps ...
        for (int kt = 0; kt < nsteps - 3; ++kt) {
            k_of_shallow(kt + 2);
            k_of_deep(kt + 3);
            SW_K_STEP(true);
        }
        // ... then the third step from the end the deep operand of the next tile's first step
        // (after the last tile: zeros) with the shallow one of this tile's last,
        k_of_shallow(nsteps - 1);
        if (have_next) begin_deep(nxt); else disable_deep();
        k_of_deep(0);
        SW_K_STEP(true);
        // the second from the end the shallow operand of the next tile's first step and the deep
        // one of its second; the next tile's epilogue values and the rows of the tile after it
        // are asked for here, ahead of this step's barrier (see pin_values) and of this tile's
        // stores,
        if (have_next) begin_shallow(nxt); else disable_shallow();
        bool have_after = false;
        if (have_next) {
            have_after = next_tile<Q_LIMITED, K_LIMITED, MODE>(a, L, L_end, stride, after);
            tile_values(nxt, tvn);
            if (GQ_ROWS && have_after) off_rows = rows_offsets(after);
        }
        k_of_shallow(0);
        k_of_deep(1);
        SW_K_STEP(true);
        // and the last one the shallow operand of its second step only: the deep stage it frees
        // is the epilogue's.
        k_of_shallow(1);
        SW_K_STEP(false);
        const int turn_stage = dst == 0 ? kDeepStages - 1 : dst - 1;   // deep stage of the step just done

        // Epilogue.  A lane holds, for q = lane%32 of each 32x32 MFMA tile, the four
        // consecutive p = 8*(r/4) + 4*(lane/32) + r%4: 8-byte pieces scattered over 32
        // rows.  Each wave therefore turns its 128 x 128 sub-tile around, 32 rows at a
        // time, through 8 KB of LDS of its own ([q][p] bf16, 16-byte chunks XOR-swizzled
        // by row) and writes whole 256-byte row segments, 16 bytes per lane.  No barrier:
        // the LDS traffic is private to the wave and in order.
        // The lane number is laundered so that the epilogue's per-lane addresses are computed
        // here, per tile, instead of being kept in registers across the k loop.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        if (MODE == MODE_ROUTER_DWR) {
            // fp32 partial sums straight from the accumulators: four consecutive p per lane
            float *Cf = a.Cf + (size_t)cur.e * a.c_batch;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q = cur.q0 + wq * 128 + j * 32 + (ln & 31);
                if (q >= cur.qlim) continue;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int p = cur.p0 + wp * 128 + i * 32 + g * 8 + ((ln >> 5) << 2);
                        if (p < a.Pdim)
                            *(float4 *)(Cf + (size_t)q * a.ldc + p) =
                                make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1],
                                            acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                    }
            }
        } else {
            char *ep = lds + turn_stage * kOpBytes64 + wave * kTurnBytes;
            bf16 *Cout = a.Cout + (size_t)cur.e * a.c_batch;
            const int c = ln & 15;
            uint32_t *bits = EPI_BASE == EPI_NONE ? nullptr : bits_of(ln);
            const int p = cur.p0 + wp * 128 + c * 8;
            // ASYNC_STORES: the tile's rows that exist as a buffer of their own, so that rows
            // past them (and, by their offset, columns past the matrix) store nothing
            i32x4 c_rsrc = {0, 0, 0, 0}, s_rsrc = {0, 0, 0, 0};
            uint32_t c_voff = 0;
            const uint32_t row_bytes = (uint32_t)a.ldc * 2u;
            if (ASYNC_STORES) {
                const int rows = cur.qlim - cur.q0 < kBQ ? cur.qlim - cur.q0 : kBQ;
                c_rsrc = make_rsrc(Cout + (size_t)cur.q0 * a.ldc, (uint32_t)rows * row_bytes);
                if (SCATTER) s_rsrc = make_rsrc(a.Cscatter, a.gather_bytes);
                c_voff = (p < a.Pdim ? (uint32_t)p * 2u : kOobOffset) +
                         (uint32_t)(wq * 128 + (ln >> 4)) * row_bytes;
            }
            // ReLU mask: byte j * 8 + i8 of a lane's 32 bytes says which of the eight
            // elements of the 16-byte piece the lane handles in round j, iteration i8 are
            // > 0.  EPI_RELU (the first forward GEMM) writes the bits, EPI_MASK (the gradient
            // w.r.t. the hidden activations, same tiling and same lane-to-element map)
            // applies them: 32 bytes per lane instead of a second read of the activations.
            uint32_t new_bits[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};   // EPI_RELU: the lane's bits of this tile
            const int wrow = ln & 31;
            // ROUTER_DX: the round's eight addend pieces, asked for before the round is turned
            // around so that their latency overlaps it
            u32x4 addend[8];
            bool has_addend[8];
            auto ask_addend = [&](int j) {
#pragma unroll
                for (int i8 = 0; i8 < 8; ++i8) {
                    const int row = j * 32 + i8 * 4 + (ln >> 4);
                    const int slot = __shfl(j < 2 ? tv.slot_lo : tv.slot_hi, row & 63);
                    has_addend[i8] = slot >= 0 && p < a.Pdim;
                    addend[i8] = u32x4{0u, 0u, 0u, 0u};
                    if (has_addend[i8]) addend[i8] = *(const u32x4 *)(a.mask + (size_t)slot * a.ldc + p);
                }
            };
            // round j, first half: the lane's accumulators of rows 32 j .. of the wave's sub-tile,
            // converted, into the turn-around buffer
            auto turn_in = [&](int j) {
                // expert dropout: the draw of hidden unit p of token t is element t * d_ff + p of
                // the dropout stream; the lane's accumulators of this round belong to one slot
                uint32_t drop_row = 0;
                if (DROP && EPI_BASE == EPI_RELU) {
                    const int tok = __shfl(j < 2 ? tv.tok_lo : tv.tok_hi, (j & 1) * 32 + wrow, kWave);
                    drop_row = (uint32_t)tok * (uint32_t)a.Pdim +
                               (uint32_t)(cur.p0 + wp * 128 + ((ln >> 5) << 2));
                }
                // the gate of the slot whose accumulators the lane holds in this round
                float row_gate = 1.f;
                if (SCALE)
                    row_gate = __uint_as_float(
                        (uint32_t)__shfl((int)(j < 2 ? tv.ep_lo : tv.ep_hi), (j & 1) * 32 + wrow, kWave));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc[i][j][g * 4 + r];
                        if (EPI_BASE == EPI_RELU) {
                            // (the ReLU itself is taken on the rounded values below: every
                            // factor applied in between is positive or zero)
                            if (DROP) {   // the lane's four units are two aligned pairs
                                const uint32_t first = drop_row + (uint32_t)(i * 32 + g * 8);
#pragma unroll
                                for (int h = 0; h < 2; ++h) {
                                    const uint32_t z = dropout_pair_bits(a.nz, (first >> 1) + (uint32_t)h);
                                    v[2 * h] = dropout_keeps_even(a.nz, z) ? v[2 * h] * a.nz.drop_scale : 0.f;
                                    v[2 * h + 1] =
                                        dropout_keeps_odd(a.nz, z) ? v[2 * h + 1] * a.nz.drop_scale : 0.f;
                                }
                            }
                        }
                        if (DROP && EPI_BASE == EPI_MASK) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] *= a.nz.drop_scale;
                        }
                        if (SCALE) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] *= row_gate;
                        }
                        uint2 o = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
                        if (EPI_BASE == EPI_RELU) {
                            // ReLU on the bf16 values, two per instruction: read as 16-bit
                            // integers the negative ones (and -0) are < 0, the others unchanged
                            o.x = pk_max_i16(o.x, 0u);
                            o.y = pk_max_i16(o.y, 0u);
                        }
                        const int ch = i * 4 + g;
                        *(uint2 *)(ep + wrow * 256 + ((ch ^ (wrow & 15)) << 4) + ((ln >> 5) << 3)) = o;
                    }
                }
            };
            // second half: the round's rows read back as 16-byte pieces of 256-byte segments.  All
            // eight are read before the first is stored (the stores are fences to the compiler,
            // which would otherwise read, wait and store in turn).
            u32x4 vals[8];
            auto turn_out = [&]() {
#pragma unroll
                for (int i8 = 0; i8 < 8; ++i8) {
                    const int rrow = i8 * 4 + (ln >> 4);
                    vals[i8] = *(const u32x4 *)(ep + rrow * 256 + ((c ^ (rrow & 15)) << 4));
                }
            };
            // third: what is left to do on the pieces, and their stores
            auto store_round = [&](int j) {
                uint32_t m_lo = 0u, m_hi = 0u;
                if (EPI_BASE == EPI_MASK) { m_lo = tv.mb[2 * j]; m_hi = tv.mb[2 * j + 1]; }
#pragma unroll
                for (int i8 = 0; i8 < 8; ++i8) {
                    const int rrow = i8 * 4 + (ln >> 4);       // row within the round
                    const int row = j * 32 + rrow;               // row within the wave's sub-tile
                    const int q = cur.q0 + row_of(wq, j, rrow);
                    u32x4 val = vals[i8];
                    uint32_t row_off = 0;   // SCATTER: the row's place (asked of the lane that holds it, by all lanes)
                    if (SCATTER) row_off = (uint32_t)__shfl((int)(j < 2 ? tv.ep_lo : tv.ep_hi), row & 63, kWave);
                    if (EPI_BASE == EPI_RELU) {
                        // After ReLU every half word is a non-negative bf16: read as an unsigned
                        // integer it is > 0 exactly when min(., 1) is 1.  Bits 0..3 of the
                        // byte: low halves of the four words, bits 4..7: high halves.
                        uint32_t u = 0;
#pragma unroll
                        for (int w = 0; w < 4; ++w) u |= pk_min_u16(val[w], 0x00010001u) << w;
                        const uint32_t byte = (u & 0xfu) | ((u >> 12) & 0xf0u);
                        if (i8 < 4) m_lo |= byte << (8 * i8);
                        else m_hi |= byte << (8 * (i8 - 4));
                    }
                    if (EPI_BASE == EPI_MASK) {
                        uint32_t byte = (i8 < 4 ? m_lo >> (8 * i8) : m_hi >> (8 * (i8 - 4))) & 0xffu;
                        byte |= byte << 12;   // bit w -> bit w, bit 4+w -> bit 16+w
#pragma unroll
                        for (int w = 0; w < 4; ++w) val[w] &= ((byte >> w) & 0x10001u) * 0xffffu;
                    }
                    if (ASYNC_STORES) {
                        store16(c_rsrc, c_voff + (uint32_t)(j * 32 + i8 * 4) * row_bytes, val);
                        // the same row, at its token's place in the token-major output
                        if (SCATTER)
                            store16(s_rsrc, p < a.Pdim ? row_off + (uint32_t)p * 2u : kOobOffset, val);
                    } else if (q < cur.qlim && p < a.Pdim) {
                        const size_t off = (size_t)q * a.ldc + p;
                        if (MODE == MODE_ROUTER_DX && has_addend[i8]) {
                            // add the token's row of the expert-side gradient (fp32 add, one rounding)
                            const bf16x8 va = __builtin_bit_cast(bf16x8, val);
                            const bf16x8 vb = __builtin_bit_cast(bf16x8, addend[i8]);
                            bf16x8 vo;
#pragma unroll
                            for (int w = 0; w < 8; ++w) vo[w] = (bf16)((float)va[w] + (float)vb[w]);
                            val = __builtin_bit_cast(u32x4, vo);
                        }
                        *(u32x4 *)(Cout + off) = val;
                    }
                }
                if (EPI_BASE == EPI_RELU) {
                    new_bits[2 * j] = m_lo;
                    new_bits[2 * j + 1] = m_hi;
                }
            };
            if (MODE == MODE_ROUTER_DX) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ask_addend(j);
                    turn_in(j);
                    turn_out();
                    store_round(j);
                }
            } else {
                // The rounds overlap: round j + 1 is converted and written into the buffer (behind
                // round j's reads, which the LDS executes in order) before round j's pieces are
                // waited for and stored, so that the conversions cover the reads' latency.
                turn_in(0);
                turn_out();
#pragma unroll
                for (int j = 1; j < 4; ++j) {
                    turn_in(j);
                    store_round(j - 1);
                    turn_out();
                }
                store_round(3);
            }
            if (EPI_BASE == EPI_RELU) {
                if (ASYNC_STORES) {
                    const i32x4 b_rsrc =
                        make_rsrc(a.relu_bits + (size_t)cur.index * kReluBitsPerTile, kReluBitsPerTile);
                    const uint32_t at = (uint32_t)(wave * 64 + ln) * 32u;
                    store16(b_rsrc, at, u32x4{new_bits[0], new_bits[1], new_bits[2], new_bits[3]});
                    store16(b_rsrc, at + 16u, u32x4{new_bits[4], new_bits[5], new_bits[6], new_bits[7]});
                } else {
                    *(u32x4 *)bits = u32x4{new_bits[0], new_bits[1], new_bits[2], new_bits[3]};
                    *(u32x4 *)(bits + 4) = u32x4{new_bits[4], new_bits[5], new_bits[6], new_bits[7]};
                }
            }
        }
        if (!have_next) break;
        // The next tile: once every wave has left its turn-around buffer, the deep operand of its
        // third step goes into that stage.  Nothing waits for the stores here.
        cur = nxt;
        nxt = after;
        have_next = have_after;
        tv = tvn;
        __syncthreads();
        k_of_deep(2);
#pragma unroll
        for (int g = 0; g < 8; ++g) SW_ISSUE_DEEP(turn_stage, g);
        first_step = true;
    }
    SW_WAIT_VMCNT(0);   // the trailing (zero) loads have landed
#undef SW_K_STEP
#undef SW_ISSUE_DEEP
#undef SW_ISSUE_SHALLOW
#undef SW_ISSUE_P_AT
#undef SW_ISSUE_Q_AT
#undef SW_P_AT
#undef SW_Q_AT
#undef SW_DEEP_AT
#undef SW_SHALLOW_AT
#undef SW_READ_GROUP
#undef SW_MFMA_PAIR
}
#undef SW_WAIT_VMCNT

// Number of CUs of the current device, rounded down to a multiple of kXcds.
static int persistent_blocks() {
    static PerDeviceOnce once;
    static int blocks[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    (void)once_per_device(once, [&] {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus < kXcds)
            cus = 256;
        blocks[dev] = cus / kXcds * kXcds;
        return hipSuccess;
    });
    return blocks[dev];
}

template <bool Q_TRANS, bool P_TRANS, int EPI, bool Q_LIMITED, bool K_LIMITED,
          int MODE = MODE_EXPERTS, int GATHER = GATHER_NONE, bool DEEP_Q = false>
static hipError_t gemm_launch(const GemmArgs &a, hipStream_t s) {
    auto kern = gemm_bf16_kernel<Q_TRANS, P_TRANS, EPI, Q_LIMITED, K_LIMITED, MODE, GATHER, DEEP_Q>;
    static PerDeviceOnce once;   // one per template instantiation
    hipError_t attr_err = once_per_device(once, [&] {
        return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kGemmLds);
    });
    if (attr_err != hipSuccess) return attr_err;
    // one block per CU (the 128 KB of LDS and 512 registers per lane allow no more)
    int blocks = persistent_blocks();
    const int needed = (int)(ceil_div(a.total_tiles, kXcds) * kXcds);
    if (needed < blocks) blocks = needed;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kGemmThreads), kGemmLds, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(GemmKind kind, const Workspace &w, char *ws, const void *W_in,
                            const void *W_out, void *dW_in, void *dW_out, const TokenMajor &tm,
                            hipStream_t s) {
    const int d = (int)w.d, f = (int)w.f, f1 = (int)w.f1, C = (int)w.C, E = (int)w.E;
    GemmArgs a{};
    a.kept = (const int32_t *)(ws + w.kept);
    const bf16 *Xd = (const bf16 *)(ws + w.Xd);
    bf16 *A = (bf16 *)(ws + w.A);
    bf16 *O = (bf16 *)(ws + w.O);
    const bf16 *dO = (const bf16 *)(ws + w.dO);
    bf16 *dH = (bf16 *)(ws + w.dH);
    bf16 *dXd = (bf16 *)(ws + w.dXd);
    auto finish = [&](int Qdim, int Pdim, int Kdim) {
        a.Qdim = Qdim; a.Pdim = Pdim; a.Kdim = Kdim;
        a.tiles_q = (int)ceil_div(Qdim, kBQ);
        a.tiles_p = (int)ceil_div(Pdim, kBP);
        a.total_tiles = a.tiles_q * a.tiles_p * E;
    };
    // With w.fused the token-major tensors take the place of the dispatched copies: x for Xd,
    // dy for dO (the gate moves into A and into the row scales), y is written by the second
    // GEMM (see the head of this file).
    const bool fused = w.fused;
    a.slot_token = (const int32_t *)(ws + w.slot_token);
    a.slots = C;
    a.row_scale = (const float *)(ws + w.slot_gate);
    a.slot_off = (const uint32_t *)(ws + w.slot_off);
    a.gather_bytes = (uint32_t)((size_t)w.T * d * 2);
    // A GEMM that follows the producer of its large activation operand walks the experts in
    // the opposite order: the producer's last-written experts are the ones still in the
    // memory-side cache (measured: 2-3 % of those kernels' time).
    a.reverse = kind == GEMM_FWD2 || kind == GEMM_DGRAD1;
    switch (kind) {
    case GEMM_FWD1: {
        a.Q = fused ? (const bf16 *)tm.x : Xd; a.q_batch = fused ? 0 : (size_t)C * d; a.ldq = d;
        a.P = (const bf16 *)W_in; a.p_batch = (size_t)d * f1; a.ldp = f1;
        a.Cout = w.geglu ? (bf16 *)(ws + w.H) : A; a.c_batch = (size_t)C * f1; a.ldc = f1;
        a.relu_bits = (uint8_t *)(ws + w.relu_bits);
        finish(C, f1, d);
        if (a.total_tiles == 0) return hipSuccess;
        if (w.geglu) {   // the plain product; activation, dropout and gate follow in geglu_fwd
            ProfScope ps("gemm1_fwd", s);
            if (fused)
                return gemm_launch<false, true, EPI_NONE, true, false, MODE_EXPERTS, GATHER_Q>(a, s);
            return gemm_launch<false, true, EPI_NONE, true, false>(a, s);
        }
        ProfScope ps("gemm1_fwd_relu", s);
        a.nz = w.noise;
        if (fused) {
            if (w.noise.dropout)
                return gemm_launch<false, true, EPI_RELU | EPI_DROP | EPI_SCALE, true, false,
                                   MODE_EXPERTS, GATHER_Q>(a, s);
            return gemm_launch<false, true, EPI_RELU | EPI_SCALE, true, false, MODE_EXPERTS,
                               GATHER_Q>(a, s);
        }
        if (w.noise.dropout)
            return gemm_launch<false, true, EPI_RELU | EPI_DROP, true, false>(a, s);
        return gemm_launch<false, true, EPI_RELU, true, false>(a, s);
    }
    case GEMM_FWD2: {
        a.Q = A; a.q_batch = (size_t)C * f; a.ldq = f;
        a.P = (const bf16 *)W_out; a.p_batch = (size_t)f * d; a.ldp = d;
        a.Cout = O; a.c_batch = (size_t)C * d; a.ldc = d;
        a.Cscatter = (bf16 *)tm.y;
        finish(C, d, f);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm2_fwd", s);
        // (both operands come from HBM here, k is long: with the activations in the deep ring the
        // CUs that share an operand tile stay close enough for the L2 -- 1.03 GB fetched instead
        // of 1.38 GB at Switch-Base -- and the kernel is 3 % faster there, 5 % at the XXL shape)
        if (fused)
            return gemm_launch<false, true, EPI_SCATTER, true, false, MODE_EXPERTS, GATHER_NONE, true>(a, s);
        return gemm_launch<false, true, EPI_NONE, true, false, MODE_EXPERTS, GATHER_NONE, true>(a, s);
    }
    case GEMM_DGRAD2: {
        a.Q = fused ? (const bf16 *)tm.dy : dO; a.q_batch = fused ? 0 : (size_t)C * d; a.ldq = d;
        a.P = (const bf16 *)W_out; a.p_batch = (size_t)f * d; a.ldp = d;   // [p = f][k = d]
        a.Cout = w.geglu ? (bf16 *)(ws + w.dA) : dH; a.c_batch = (size_t)C * f; a.ldc = f;
        a.relu_bits = (uint8_t *)(ws + w.relu_bits);
        finish(C, f, d);
        if (a.total_tiles == 0) return hipSuccess;
        a.nz = w.noise;
        if (w.geglu) {
            ProfScope ps("gemm2_dgrad", s);
            if (fused)
                return gemm_launch<false, false, EPI_SCALE, true, false, MODE_EXPERTS, GATHER_Q>(a, s);
            return gemm_launch<false, false, EPI_NONE, true, false>(a, s);
        }
        ProfScope ps("gemm2_dgrad_relumask", s);
        if (fused) {
            if (w.noise.dropout)
                return gemm_launch<false, false, EPI_MASK | EPI_DROP | EPI_SCALE, true, false,
                                   MODE_EXPERTS, GATHER_Q>(a, s);
            return gemm_launch<false, false, EPI_MASK | EPI_SCALE, true, false, MODE_EXPERTS,
                               GATHER_Q>(a, s);
        }
        if (w.noise.dropout)
            return gemm_launch<false, false, EPI_MASK | EPI_DROP, true, false>(a, s);
        return gemm_launch<false, false, EPI_MASK, true, false>(a, s);
    }
    case GEMM_DGRAD1: {
        a.Q = dH; a.q_batch = (size_t)C * f1; a.ldq = f1;
        a.P = (const bf16 *)W_in; a.p_batch = (size_t)d * f1; a.ldp = f1;    // [p = d][k = f1]
        a.Cout = dXd; a.c_batch = (size_t)C * d; a.ldc = d;
        finish(C, d, f1);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm1_dgrad", s);
        // (with the deep ring on Q, as in the second forward GEMM, this one also fetches 1.03
        // instead of 1.33 GB at Switch-Base, but takes 1 % longer there and 4-6 % longer on
        // the other model shapes)
        return gemm_launch<false, false, EPI_NONE, true, false>(a, s);
    }
    case GEMM_WGRAD2: {
        a.Q = A; a.q_batch = (size_t)C * f; a.ldq = f;      // [k = slot][q = f]
        a.P = fused ? (const bf16 *)tm.dy : dO;             // [k = slot][p = d]
        a.p_batch = fused ? 0 : (size_t)C * d; a.ldp = d;
        a.Cout = (bf16 *)dW_out; a.c_batch = (size_t)f * d; a.ldc = d;
        finish(f, d, C);
        ProfScope ps("gemm2_wgrad", s);
        if (fused)
            return gemm_launch<true, true, EPI_NONE, false, true, MODE_EXPERTS, GATHER_P, true>(a, s);
        return gemm_launch<true, true, EPI_NONE, false, true, MODE_EXPERTS, GATHER_NONE, true>(a, s);
    }
    case GEMM_WGRAD1: {
        a.Q = fused ? (const bf16 *)tm.x : Xd;              // [k = slot][q = d]
        a.q_batch = fused ? 0 : (size_t)C * d; a.ldq = d;
        a.P = dH; a.p_batch = (size_t)C * f1; a.ldp = f1;     // [k = slot][p = f1]
        a.Cout = (bf16 *)dW_in; a.c_batch = (size_t)d * f1; a.ldc = f1;
        finish(d, f1, C);
        ProfScope ps("gemm1_wgrad", s);
        if (fused)
            return gemm_launch<true, true, EPI_NONE, false, true, MODE_EXPERTS, GATHER_Q>(a, s);
        return gemm_launch<true, true, EPI_NONE, false, true>(a, s);
    }
    }
    return hipErrorInvalidValue;
}

// dx = dl W_r^T + (kept) dXd[slot]: dl as bf16 hi|lo rows [tile][T][256], W_r^T as bf16 hi|lo
// rows [tile][d][256], one plane per tile of 128 experts; see GemmMode.  With input jitter the product alone is written (no token has an
// addend row); router_dx_jitter_kernel then scales it by the multipliers and adds the rows.
hipError_t launch_router_dx_mfma(const Workspace &w, char *ws, void *dx, hipStream_t s) {
    GemmArgs a{};
    a.Q = (const bf16 *)(ws + w.dl_split); a.q_batch = 0; a.ldq = 256;
    a.P = (const bf16 *)(ws + w.wsplit_b); a.p_batch = 0; a.ldp = 256;
    a.Cout = (bf16 *)dx; a.c_batch = 0; a.ldc = (int)w.d;
    a.mask = (const bf16 *)(ws + w.dXd);
    a.tok_slot = (const int32_t *)(ws + (w.noise.jitter ? w.no_slot : w.tok_slot));
    a.router_tiles = (int)w.etiles;
    a.q_plane = (int)(w.T * 256);
    a.p_plane = (int)(w.d * 256);
    a.Qdim = (int)w.T; a.Pdim = (int)w.d; a.Kdim = 384 * (int)w.etiles;
    a.tiles_q = (int)ceil_div(a.Qdim, kBQ);
    a.tiles_p = (int)ceil_div(a.Pdim, kBP);
    a.total_tiles = a.tiles_q * a.tiles_p;
    ProfScope ps("router_dx_mfma", s);
    return gemm_launch<false, false, EPI_NONE, false, false, MODE_ROUTER_DX>(a, s);
}

// Partial sums over token ranges of x^T [dl_hi | dl_lo]  ->  part[split][d][256] (fp32).
// With input jitter x is replaced by the hi and mid planes of x * m, taken as one operand of
// 2 dpad rows: part[split][2 dpad][256], row k from the hi plane, row dpad + k from the mid plane.
hipError_t launch_router_dWr_mfma(const Workspace &w, const void *x, char *ws, hipStream_t s) {
    const bool jitter = w.noise.jitter;
    const int ldx = jitter ? (int)w.dpad_r : (int)w.d;
    const int rows = jitter ? 2 * (int)w.dpad : (int)w.d;
    ProfScope ps("router_dWr_mfma", s);
    // one launch per tile of 128 experts: part[tile][split][rows][256]
    for (int tile = 0; tile < (int)w.etiles; ++tile) {
        GemmArgs a{};
        a.Q = jitter ? (const bf16 *)(ws + w.xj) : (const bf16 *)x;                  // [k = token][q]
        a.q_batch = (size_t)w.tps_m * ldx; a.ldq = ldx;
        a.P = (const bf16 *)(ws + w.dl_split) + (size_t)tile * w.T * 256;           // [k = token][p]
        a.p_batch = (size_t)w.tps_m * 256; a.ldp = 256;
        a.Cf = (float *)(ws + w.dWr_part_m) + (size_t)tile * w.nsplit_m * rows * 256;
        a.c_batch = (size_t)rows * 256; a.ldc = 256;
        a.T_total = (int)w.T; a.tps = (int)w.tps_m;
        a.Qdim = rows; a.Pdim = 256; a.Kdim = (int)w.tps_m;
        a.tiles_q = (int)ceil_div(a.Qdim, kBQ);
        a.tiles_p = 1;
        a.total_tiles = a.tiles_q * a.tiles_p * (int)w.nsplit_m;
        hipError_t err = gemm_launch<true, true, EPI_NONE, false, true, MODE_ROUTER_DWR>(a, s);
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

}  // namespace sw
