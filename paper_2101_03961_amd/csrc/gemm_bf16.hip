// Grouped expert GEMMs on bf16 MFMA (gfx950), fp32 accumulation.
//
// For every expert e the kernel computes a tile of
//     C_e[q][p] = sum_k Q_e(q,k) * P_e(p,k)          (C row-major, p contiguous)
// with a 256 (p) x 256 (q) x 64 (k) block tile, four wavefronts in a 2 x 2
// arrangement, each owning a 128 x 128 sub-tile as 4 x 4 MFMA 32x32x16 tiles
// (256 fp32 accumulators per lane).  Both operand tiles are staged in LDS as
// [row][64 k] with k contiguous, which is what the MFMA operand registers want
// (8 consecutive k per lane); an operand whose memory layout is k-major
// ([k][row], row contiguous -- the weights in the forward pass, both operands
// of the weight-gradient GEMMs) is transposed in registers, 8x8 elements per
// lane, between the global load and the LDS store.  P feeds the MFMA "A" side,
// so each lane ends up with four consecutive p of one q and stores 8 bytes.
//
// LDS is double buffered (2 x 64 KB): one barrier per k step, global loads for
// step i+1 are in flight while step i is multiplied.
//
// Work assignment: one block per (expert, p tile, q tile); q tiles beyond the
// expert's kept-token count exit at once.  Block ids are spread so that the
// tiles of one expert land on the same XCD (and its L2) next to each other.
#include "common.h"

namespace sw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBP = 256;        // block tile, p rows
constexpr int kBQ = 256;        // block tile, q rows
constexpr int kBK = 64;         // k per step
constexpr int kGemmThreads = 256;
constexpr int kTileBytes = kBP * kBK * 2;          // 32 KB per operand tile
constexpr int kStageBytes = 2 * kTileBytes;        // P + Q
constexpr int kGemmLds = 2 * kStageBytes;          // double buffered: 128 KB
constexpr int kXcds = 8;

struct GemmArgs {
    const bf16 *Q;      // per expert: q_batch elements
    const bf16 *P;
    bf16 *Cout;
    const bf16 *mask;   // same layout as Cout (ReLU mask source) or nullptr
    size_t q_batch, p_batch, c_batch;
    int ldq, ldp, ldc;  // leading dimensions in elements
    int Qdim, Pdim, Kdim;
    const int32_t *kept;
    int tiles_q, tiles_p, total_tiles;
};

// 16-byte chunk position inside a [row][64 k] LDS tile, XOR-swizzled so that
// both the MFMA operand reads (32 consecutive rows, one chunk column) and the
// transposing stores (rows 8 apart) spread over all banks.
__device__ __forceinline__ int lds_off(int row, int kc) {
    return row * (kBK * 2) + (((kc ^ (row + (row >> 3))) & 7) << 4);
}

struct Stage {
    uint4 v[8];
};

// Operand stored [row][k], k contiguous: thread loads 8 chunks (row = id/8, kc = id%8).
__device__ __forceinline__ void load_direct(Stage &st, const bf16 *base, int ld, int row0,
                                            int rowlim, int k0, int klim, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = i * kGemmThreads + tid;
        const int row = row0 + (id >> 3);
        const int k = k0 + ((id & 7) << 3);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < rowlim && k < klim) v = *(const uint4 *)(base + (size_t)row * ld + k);
        st.v[i] = v;
    }
}
__device__ __forceinline__ void store_direct(const Stage &st, char *tile, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = i * kGemmThreads + tid;
        *(uint4 *)(tile + lds_off(id >> 3, id & 7)) = st.v[i];
    }
}

// Operand stored [k][row], row contiguous: thread loads an 8 (k) x 8 (row) block.
__device__ __forceinline__ void load_trans(Stage &st, const bf16 *base, int ld, int row0,
                                           int rowlim, int k0, int klim, int tid) {
    const int kg = tid >> 5;          // 0..7
    const int rc = tid & 31;          // 0..31
    const int row = row0 + (rc << 3);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = k0 + (kg << 3) + j;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < rowlim && k < klim) v = *(const uint4 *)(base + (size_t)k * ld + row);
        st.v[j] = v;
    }
}
__device__ __forceinline__ void store_trans(const Stage &st, char *tile, int tid) {
    const int kg = tid >> 5;
    const int rc = tid & 31;
    const uint32_t *w = (const uint32_t *)st.v;   // w[j*4 + c2]: row j, elements 2c2, 2c2+1
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int c2 = c >> 1;
        uint32_t o[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t lo = w[(2 * m) * 4 + c2];
            const uint32_t hi = w[(2 * m + 1) * 4 + c2];
            o[m] = (c & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
        }
        *(uint4 *)(tile + lds_off((rc << 3) + c, kg)) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

enum { EPI_NONE = 0, EPI_RELU = 1, EPI_MASK = 2 };

template <bool Q_TRANS, bool P_TRANS, int EPI, bool Q_LIMITED, bool K_LIMITED>
__global__ __launch_bounds__(kGemmThreads) void gemm_bf16_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wp = wave & 1;
    const int wq = wave >> 1;

    // block id -> tile, keeping one expert's tiles on one XCD
    const int per_xcd = gridDim.x / kXcds;
    const int L = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (L >= a.total_tiles) return;
    const int tiles_pe = a.tiles_q * a.tiles_p;
    const int e = L / tiles_pe;
    const int rem = L - e * tiles_pe;
    const int pt = rem / a.tiles_q;
    const int qt = rem - pt * a.tiles_q;
    const int p0 = pt * kBP;
    const int q0 = qt * kBQ;

    const int kept = a.kept[e];
    const int qlim = Q_LIMITED ? (kept < a.Qdim ? kept : a.Qdim) : a.Qdim;
    const int klim = K_LIMITED ? (kept < a.Kdim ? kept : a.Kdim) : a.Kdim;
    if (q0 >= qlim) return;

    const bf16 *Q = a.Q + (size_t)e * a.q_batch;
    const bf16 *P = a.P + (size_t)e * a.p_batch;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (klim + kBK - 1) / kBK;
    Stage sp, sq;
    if (nk > 0) {
        if (P_TRANS) load_trans(sp, P, a.ldp, p0, a.Pdim, 0, klim, tid);
        else load_direct(sp, P, a.ldp, p0, a.Pdim, 0, klim, tid);
        if (Q_TRANS) load_trans(sq, Q, a.ldq, q0, qlim, 0, klim, tid);
        else load_direct(sq, Q, a.ldq, q0, qlim, 0, klim, tid);
    }
    for (int kt = 0; kt < nk; ++kt) {
        char *tp = lds + (kt & 1) * kStageBytes;
        char *tq = tp + kTileBytes;
        if (P_TRANS) store_trans(sp, tp, tid); else store_direct(sp, tp, tid);
        if (Q_TRANS) store_trans(sq, tq, tid); else store_direct(sq, tq, tid);
        __syncthreads();
        if (kt + 1 < nk) {
            const int k0 = (kt + 1) * kBK;
            if (P_TRANS) load_trans(sp, P, a.ldp, p0, a.Pdim, k0, klim, tid);
            else load_direct(sp, P, a.ldp, p0, a.Pdim, k0, klim, tid);
            if (Q_TRANS) load_trans(sq, Q, a.ldq, q0, qlim, k0, klim, tid);
            else load_direct(sq, Q, a.ldq, q0, qlim, k0, klim, tid);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int kc = ks * 2 + (lane >> 5);
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                fa[i] = *(const bf16x8 *)(tp + lds_off(wp * 128 + i * 32 + (lane & 31), kc));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                fb[j] = *(const bf16x8 *)(tq + lds_off(wq * 128 + j * 32 + (lane & 31), kc));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue: lane holds, for q = lane%32 of each 32x32 tile, p = 8*(r/4) + 4*(lane/32) + r%4
    bf16 *Cout = a.Cout + (size_t)e * a.c_batch;
    const bf16 *mask = EPI == EPI_MASK ? a.mask + (size_t)e * a.c_batch : nullptr;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = q0 + wq * 128 + j * 32 + (lane & 31);
        if (q >= qlim) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int p = p0 + wp * 128 + i * 32 + g * 8 + ((lane >> 5) << 2);
                if (p >= a.Pdim) continue;
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = acc[i][j][g * 4 + r];
                if (EPI == EPI_RELU) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
                }
                if (EPI == EPI_MASK) {
                    const bf16x4 m = *(const bf16x4 *)(mask + (size_t)q * a.ldc + p);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = (float)m[r] > 0.f ? v[r] : 0.f;
                }
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (bf16)v[r];
                *(bf16x4 *)(Cout + (size_t)q * a.ldc + p) = o;
            }
        }
    }
}

template <bool Q_TRANS, bool P_TRANS, int EPI, bool Q_LIMITED, bool K_LIMITED>
static hipError_t gemm_launch(const GemmArgs &a, int E, hipStream_t s) {
    auto kern = gemm_bf16_kernel<Q_TRANS, P_TRANS, EPI, Q_LIMITED, K_LIMITED>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t err = hipFuncSetAttribute((const void *)kern,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (err != hipSuccess) return err;
        attr_set = true;
    }
    const int64_t blocks = ceil_div(a.total_tiles, kXcds) * kXcds;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kGemmThreads), kGemmLds, s, a);
    (void)E;
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(GemmKind kind, const Workspace &w, char *ws, const void *W_in,
                            const void *W_out, void *dW_in, void *dW_out, hipStream_t s) {
    const int d = (int)w.d, f = (int)w.f, C = (int)w.C, E = (int)w.E;
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
    switch (kind) {
    case GEMM_FWD1: {
        a.Q = Xd; a.q_batch = (size_t)C * d; a.ldq = d;
        a.P = (const bf16 *)W_in; a.p_batch = (size_t)d * f; a.ldp = f;
        a.Cout = A; a.c_batch = (size_t)C * f; a.ldc = f;
        finish(C, f, d);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm1_fwd_relu", s);
        return gemm_launch<false, true, EPI_RELU, true, false>(a, E, s);
    }
    case GEMM_FWD2: {
        a.Q = A; a.q_batch = (size_t)C * f; a.ldq = f;
        a.P = (const bf16 *)W_out; a.p_batch = (size_t)f * d; a.ldp = d;
        a.Cout = O; a.c_batch = (size_t)C * d; a.ldc = d;
        finish(C, d, f);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm2_fwd", s);
        return gemm_launch<false, true, EPI_NONE, true, false>(a, E, s);
    }
    case GEMM_DGRAD2: {
        a.Q = dO; a.q_batch = (size_t)C * d; a.ldq = d;
        a.P = (const bf16 *)W_out; a.p_batch = (size_t)f * d; a.ldp = d;   // [p = f][k = d]
        a.Cout = dH; a.c_batch = (size_t)C * f; a.ldc = f; a.mask = A;
        finish(C, f, d);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm2_dgrad_relumask", s);
        return gemm_launch<false, false, EPI_MASK, true, false>(a, E, s);
    }
    case GEMM_DGRAD1: {
        a.Q = dH; a.q_batch = (size_t)C * f; a.ldq = f;
        a.P = (const bf16 *)W_in; a.p_batch = (size_t)d * f; a.ldp = f;    // [p = d][k = f]
        a.Cout = dXd; a.c_batch = (size_t)C * d; a.ldc = d;
        finish(C, d, f);
        if (a.total_tiles == 0) return hipSuccess;
        ProfScope ps("gemm1_dgrad", s);
        return gemm_launch<false, false, EPI_NONE, true, false>(a, E, s);
    }
    case GEMM_WGRAD2: {
        a.Q = A; a.q_batch = (size_t)C * f; a.ldq = f;      // [k = slot][q = f]
        a.P = dO; a.p_batch = (size_t)C * d; a.ldp = d;     // [k = slot][p = d]
        a.Cout = (bf16 *)dW_out; a.c_batch = (size_t)f * d; a.ldc = d;
        finish(f, d, C);
        ProfScope ps("gemm2_wgrad", s);
        return gemm_launch<true, true, EPI_NONE, false, true>(a, E, s);
    }
    case GEMM_WGRAD1: {
        a.Q = Xd; a.q_batch = (size_t)C * d; a.ldq = d;     // [k = slot][q = d]
        a.P = dH; a.p_batch = (size_t)C * f; a.ldp = f;     // [k = slot][p = f]
        a.Cout = (bf16 *)dW_in; a.c_batch = (size_t)d * f; a.ldc = f;
        finish(d, f, C);
        ProfScope ps("gemm1_wgrad", s);
        return gemm_launch<true, true, EPI_NONE, false, true>(a, E, s);
    }
    }
    return hipErrorInvalidValue;
}

}  // namespace sw
