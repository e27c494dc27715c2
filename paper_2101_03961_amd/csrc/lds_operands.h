// MFMA operand staging shared by the grouped expert GEMM and the router kernels
// (gfx950): direct global -> LDS loads, LDS tile layouts, fragment reads.
#pragma once

#include "common.h"

namespace sw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kOpBytes = 256 * 32 * 2;   // one 256-row x 32-k bf16 operand stage: 16 KB

// Offset used by lanes that must read zeros: beyond every descriptor (all
// descriptors are kept below 2 GB by the host-side shape check).
constexpr uint32_t kOobOffset = 0x80000000u;

// Raw buffer descriptor: base, stride 0, size in bytes, 32-bit data format.
__device__ __forceinline__ i32x4 make_rsrc(const void *base, uint32_t bytes) {
    const uint64_t a = (uint64_t)base;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One direct global -> LDS load of 16 bytes per lane: lane l's bytes land at
// LDS offset lds_base + 16 l.  lds_base and soff are wave-uniform.  The s_nop covers two
// hazards the compiler does not see inside asm: m0 written one state before the load, and a
// descriptor or offset register reloaded from a spill lane (v_readlane) fewer than five
// states before it.
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 3\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// ---- operand stored [row][k], k contiguous ---------------------------------------
// LDS stage layout: [256 rows][32 k] = 64 bytes per row, four 16-byte chunks,
// chunk c of row r kept at position c ^ dswz(r).  dswz uses row bits 1..3, so
// that 8 (or 16) consecutive rows reading the same logical chunk touch every
// bank once whether the LDS cycles 128 or 256 bytes.
__device__ __forceinline__ int dswz(int row) {
    return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}

struct DirectOperand {
    i32x4 rsrc;
    uint32_t voff;       // byte offset of the lane's chunk in the wave's first 16 rows
    uint32_t row_step;   // bytes of 64 rows
    int c8;              // first k (within the step) of the lane's chunk
    int klim;
    uint32_t frag0;      // LDS byte offset (within an operand stage) of the lane's fragment, sub-step 0

    // wave_rows: first row (0 or 128) of the wave's 128-row half of the tile
    __device__ __forceinline__ void init(const bf16 *base, int ld, int row0, int rowlim, int klim_,
                                         int lane, int wave, int wave_rows) {
        rsrc = make_rsrc(base, (uint32_t)rowlim * (uint32_t)ld * 2u);
        const int r = wave * 16 + (lane >> 2);          // + 64 per load
        const int c = (lane & 3) ^ dswz(r);
        c8 = c << 3;
        voff = ((uint32_t)(row0 + r) * (uint32_t)ld + (uint32_t)c8) * 2u;
        row_step = 64u * (uint32_t)ld * 2u;
        klim = klim_;
        const int fr = wave_rows + (lane & 31);
        frag0 = (uint32_t)(fr * 64 + (((lane >> 5) ^ dswz(fr)) << 4));
    }
    static constexpr int kPieces = 4;   // LDS reads per k sub-step: one per fragment
    // load i of four: rows 64 i + [16 wave, 16 wave + 16)
    __device__ __forceinline__ void issue_one(uint32_t lds_op, int k0, int wave, int i) const {
        const uint32_t vo = (k0 + c8 < klim) ? voff : kOobOffset;
        dma16(rsrc, vo, (uint32_t)i * row_step + (uint32_t)k0 * 2u,
              lds_op + (uint32_t)((i * 64 + wave * 16) * 64));
    }
    // fragment x (rows 32 x .. of the rows this operand was initialised for), sub-step ks
    __device__ __forceinline__ bf16x8 read_frag(const char *lds_op, int x, int ks) const {
        return *(const bf16x8 *)(lds_op + ((frag0 ^ (uint32_t)(ks << 5)) + (uint32_t)(x * 32 * 64)));
    }
    // piece x = fragment x (rows 32 x ..), k sub-step ks (0/1): chunk 2 ks + lane/32
    __device__ __forceinline__ void read_piece(const char *lds_op, int x, int ks,
                                               s16x4 (&h)[4][2]) const {
        const s16x8 v =
            *(const s16x8 *)(lds_op + ((frag0 ^ (uint32_t)(ks << 5)) + (uint32_t)(x * 32 * 64)));
        h[x][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
        h[x][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
    }
};

// =============================================================================
// 64-k variants (one pipeline step = 64 k): an operand row of a [row][k] tile is a
// whole 128-byte line, so every request the loads make is a full cache line.
// =============================================================================
constexpr int kOpBytes64 = 256 * 64 * 2;   // 32 KB per operand stage

// [row][k] operand: LDS [256 rows][64 k] = 128 bytes per row, eight 16-byte chunks,
// chunk c of row r at position c ^ ((r >> 1) & 7): 16 consecutive rows reading the
// same logical chunk cover all 64 banks.
struct DirectOperand64 {
    i32x4 rsrc;
    uint32_t voff;       // byte offset of the lane's chunk in the wave's first 8 rows
    uint32_t row_step;   // bytes of 32 rows
    int c8;              // first k (within the step) of the lane's chunk
    int klim;
    uint32_t frag0;      // LDS byte offset of the lane's fragment, sub-step 0

    // load side: point at rows [row0, ...) of a [rowlim][ld] matrix, k < klim_
    __device__ __forceinline__ void init_load(const bf16 *base, int ld, int row0, int rowlim,
                                              int klim_, int lane, int wave) {
        rsrc = make_rsrc(base, (uint32_t)rowlim * (uint32_t)ld * 2u);
        const int r = wave * 8 + (lane >> 3);           // + 32 per load
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        c8 = c << 3;
        voff = ((uint32_t)(row0 + r) * (uint32_t)ld + (uint32_t)c8) * 2u;
        row_step = 32u * (uint32_t)ld * 2u;
        klim = klim_;
    }
    // every load reads zeros from now on
    __device__ __forceinline__ void disable_load() { klim = 0; }
    // read side: wave_rows = first row (0 or 128) of the wave's half of the tile
    __device__ __forceinline__ void init_frag(int lane, int wave_rows) {
        const int fr = wave_rows + (lane & 31);
        frag0 = (uint32_t)(fr * 128 + (((lane >> 5) ^ ((fr >> 1) & 7)) << 4));
    }
    static constexpr int kPieces = 4;   // LDS reads per k sub-step: one per fragment
    // load i of eight: rows 32 i + [8 wave, 8 wave + 8)
    __device__ __forceinline__ void issue_one(uint32_t lds_op, int k0, int wave, int i) const {
        const uint32_t vo = (k0 + c8 < klim) ? voff : kOobOffset;
        dma16(rsrc, vo, (uint32_t)i * row_step + (uint32_t)k0 * 2u,
              lds_op + (uint32_t)((i * 32 + wave * 8) * 128));
    }
    // piece x = fragment x (rows 32 x ..), k sub-step ks (0..3): chunk 2 ks + lane/32
    __device__ __forceinline__ void read_piece(const char *lds_op, int x, int ks,
                                               s16x4 (&h)[4][2]) const {
        const s16x8 v =
            *(const s16x8 *)(lds_op + ((frag0 ^ (uint32_t)(ks << 5)) + (uint32_t)(x * 32 * 128)));
        h[x][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
        h[x][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
    }
};

// The same operand with its rows gathered: tile row r is the row at byte offset off(r) of a
// token-major matrix (the dispatch of Sec. 5.4 done by the load addresses).  The eight loads of
// a lane go to eight different tokens, so their byte offsets are kept per load.
struct DirectGather64 : DirectOperand64 {
    uint32_t gvoff[8];   // byte offset of the lane's chunk for load i (>= kOobOffset: row absent)

    // off_of_lane: row offset of tile row 8 wave + (lane & 7) + 32 (lane >> 3), kOobOffset past the rows
    __device__ __forceinline__ void init_gather(const bf16 *base, uint32_t bytes, int klim_,
                                                int lane, int wave, uint32_t off_of_lane) {
        rsrc = make_rsrc(base, bytes);
        const int r = wave * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        c8 = c << 3;
        klim = klim_;
#pragma unroll
        for (int i = 0; i < 8; ++i)   // load i covers rows 32 i + 8 wave + lane / 8
            gvoff[i] = (uint32_t)__shfl((int)off_of_lane, (lane >> 3) + 8 * i, kWave) + (uint32_t)c8 * 2u;
    }
    __device__ __forceinline__ void disable_load() { klim = 0; }
    __device__ __forceinline__ void issue_one(uint32_t lds_op, int k0, int wave, int i) const {
        const uint32_t vo = (k0 + c8 < klim) ? gvoff[i] : kOobOffset;
        dma16(rsrc, vo, (uint32_t)k0 * 2u, lds_op + (uint32_t)((i * 32 + wave * 8) * 128));
    }
};

// [k][row] operand (row contiguous): LDS [64 k][256 rows] = 512 bytes per k-row, 32 chunks
// of 8 rows; chunk c of k-row k is kept at position c ^ 4 (k mod 4).  One transposing read
// (ds_read_b64_tr_b16) has lanes 0..31 fetch 64 bytes (rows 0..31 of the fragment) from each
// of four consecutive k-rows; 512 bytes apart they would all fall on the same banks, the
// permutation puts them into the four different quarters of the 256-byte bank window.
// Lanes form groups of 16; group g covers rows 16 (g&1) .. +16 of the fragment and
// k 8 (g>>1) .. +8; inside a group lane j supplies the 8 bytes at k-row j/4, rows
// 4 (j%4) .. +4, and receives k-rows 0..3 of row j.
struct TransOperand64 {
    i32x4 rsrc;
    uint32_t voff[2];       // lane's byte offset for loads with even / odd index
    uint32_t k_step;        // bytes of one k row
    uint32_t frag_base[4];  // LDS byte offset of the lane's share of fragment i (ks = 0, first half)

    __device__ __forceinline__ void init_load(const bf16 *base, int ld, int row0, int rowlim,
                                              int klim, int lane, int wave) {
        rsrc = make_rsrc(base, (uint32_t)klim * (uint32_t)ld * 2u);
        k_step = (uint32_t)ld * 2u;
        const int kk = lane >> 5, pc = lane & 31;
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            const int kr = wave * 16 + 2 * par + kk;    // loads par, par + 2, ...: same k mod 4
            const int c = pc ^ ((kr & 3) << 2);
            const int row = row0 + (c << 3);
            voff[par] = row < rowlim
                            ? ((uint32_t)(wave * 16 + kk) * (uint32_t)ld + (uint32_t)row) * 2u
                            : kOobOffset;
        }
    }
    __device__ __forceinline__ void disable_load() { voff[0] = voff[1] = kOobOffset; }
    __device__ __forceinline__ void init_frag(int lane, int wave_rows) {
        const int g = lane >> 4, j = lane & 15;
        const int kq = j >> 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = wave_rows + i * 32 + (g & 1) * 16 + (j & 3) * 4;
            const int chunk = (n >> 3) ^ (kq << 2);
            frag_base[i] = (uint32_t)((((g >> 1) * 8 + kq) * 512) + (chunk << 4) + ((n & 4) << 1));
        }
    }
    static constexpr int kPieces = 8;   // LDS reads per k sub-step: two per fragment
    // load i of eight: k-rows 16 wave + 2 i + {0, 1}
    __device__ __forceinline__ void issue_one(uint32_t lds_op, int k0, int wave, int i) const {
        dma16(rsrc, voff[i & 1], (uint32_t)(k0 + 2 * i) * k_step,
              lds_op + (uint32_t)((wave * 16 + 2 * i) * 512));
    }
    __device__ __forceinline__ void read_piece(const char *lds_op, int x, int ks,
                                               s16x4 (&h)[4][2]) const {
        typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
        const char *p0 = lds_op + frag_base[x >> 1] + ks * (16 * 512) + (x & 1) * (4 * 512);
        h[x >> 1][x & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0));
    }
};

// The same operand with its k-rows gathered: k-row k of the tile is the row at byte offset
// off(k) of a token-major matrix; issue_one is handed the offset of the k-row the lane
// fetches (kOobOffset past the tile's k range: the offset table holds that value in every
// slot without a token).  (A sum of two absent parts may wrap into the matrix: such a chunk
// lies in a column past the operand's rows, whose products are never stored.)
struct TransGather64 : TransOperand64 {
    uint32_t cvoff[2];   // byte offset of the lane's chunk inside a row, loads with even / odd index

    __device__ __forceinline__ void init_gather(const bf16 *base, uint32_t bytes, int row0,
                                                int rowlim, int lane, int wave) {
        rsrc = make_rsrc(base, bytes);
        const int kk = lane >> 5, pc = lane & 31;
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            const int kr = wave * 16 + 2 * par + kk;
            const int c = pc ^ ((kr & 3) << 2);
            const int row = row0 + (c << 3);
            cvoff[par] = row < rowlim ? (uint32_t)row * 2u : kOobOffset;
        }
    }
    __device__ __forceinline__ void disable_load() { cvoff[0] = cvoff[1] = kOobOffset; }
    // load i of eight: k-rows 16 wave + 2 i + {0, 1} of the step; row_off: the lane's k-row
    __device__ __forceinline__ void issue_one(uint32_t lds_op, int wave, int i,
                                              uint32_t row_off) const {
        dma16(rsrc, row_off + cvoff[i & 1], 0u, lds_op + (uint32_t)((wave * 16 + 2 * i) * 512));
    }
};

}  // namespace sw
