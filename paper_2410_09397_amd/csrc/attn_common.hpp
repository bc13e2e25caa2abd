// Shared device helpers for the gfx950 attention kernels: vector types, the LDS tile
// layout, MFMA operand fetches and bf16 packing.  HIP device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define ATTN_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kThreads = 256;  // four 64-lane wavefronts per workgroup, one per SIMD

// ---------------------------------------------------------------------------------------
// 32x32x16 bf16 MFMA.  Operand layout (lane l, h = l / 32):
//   A (32 x 16): row l % 32, k = 8h .. 8h+7        B (16 x 32): column l % 32, k = 8h .. 8h+7
//   C (32 x 32): column l % 32, register i <-> row 8 (i / 4) + 4h + i % 4
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of accumulator register i for a lane in half h.
__device__ __forceinline__ int acc_row(int i, int h) { return 8 * (i >> 2) + 4 * h + (i & 3); }

// Two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// Registers 8s .. 8s+7 of an accumulator as one bf16 B operand.  Its k index (h, t) then
// stands for accumulator row 16s + 8 (t / 4) + 4h + t % 4, which load_frag_t() mirrors.
__device__ __forceinline__ bf16x8 acc_to_operand(const f32x16& c, int s) {
    u32x4 r;
    r[0] = pack_bf16(c[8 * s + 0], c[8 * s + 1]);
    r[1] = pack_bf16(c[8 * s + 2], c[8 * s + 3]);
    r[2] = pack_bf16(c[8 * s + 4], c[8 * s + 5]);
    r[3] = pack_bf16(c[8 * s + 6], c[8 * s + 7]);
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ float max3(float a, float b, float c) {
    return __builtin_elementwise_maximum(a, __builtin_elementwise_maximum(b, c));
}

// ---------------------------------------------------------------------------------------
// LDS tile: R rows of D bf16, row-major, no padding, 16-byte chunks XOR-swizzled by row so
// that both fetch patterns below spread over all 64 banks:
//   - row-major fetch: 16 lanes read the same chunk column of 16 consecutive rows,
//   - transposed fetch: 32 lanes read 4 consecutive rows x 4 consecutive chunks.
// ---------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int swz(int row) {
    if constexpr (D >= 128)
        return ((row & 3) << 2) | ((row >> 2) & 3);
    else if constexpr (D == 64)
        return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    else  // D == 32: four chunks per row, only the row-major fetch is used
        return (row >> 2) & 3;
}

// Byte offset of 16-byte chunk c (8 elements) of a tile row.
template <int D>
__device__ __forceinline__ int tile_off(int row, int c) {
    return row * (D * 2) + ((c ^ swz<D>(row)) << 4);
}

// A (or B) operand whose k index runs along the tile's contiguous dimension:
// lane l holds row row0 + l % 32, elements 16 ks + 8h .. +7.
template <int D>
__device__ __forceinline__ bf16x8 load_frag(const char* tile, int row0, int ks, int lane) {
    const int row = row0 + (lane & 31);
    return *reinterpret_cast<const bf16x8*>(tile + tile_off<D>(row, 2 * ks + (lane >> 5)));
}

// A operand whose k index runs along the tile's rows (the tile is read transposed):
// lane l holds column col0 + l % 32 and, for t = 0..7, row row16 + 8 (t / 4) + 4h + t % 4.
// Two ds_read_b64_tr_b16: within each group of 16 lanes, lane s supplies the address of
// row + s / 4, columns 4 (s % 4) .. +3, and receives column s of the four rows.
template <int D>
__device__ __forceinline__ bf16x8 load_frag_t(const char* tile, int col0, int row16, int lane) {
    const int s = lane & 15;
    const int row = row16 + 4 * (lane >> 5) + (s >> 2);
    const int col = col0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int off0 = tile_off<D>(row, col >> 3) + ((col & 4) << 1);
    const int off1 = tile_off<D>(row + 8, col >> 3) + ((col & 4) << 1);
    i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(tile + off0));
    i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(tile + off1));
    typedef short i16x8 __attribute__((ext_vector_type(8)));
    i16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// The same two fetches with the lane-dependent part of the address hoisted out of the hot
// loop.  The swizzle is an XOR on the chunk field (bits 4..7 of the byte offset), tiles start on
// 256-byte boundaries and rows that are a multiple of 16 apart share their swizzle term, so
//   offset(ks)  = (tile + rm0) ^ (ks << 5)            + row0 * row_bytes      (load_frag)
//   offset(mt)  = (tile + tr0) ^ (mt << 6) [^ 32 for the rows + 8 half] + ...  (load_frag_t)
// i.e. one per-lane base per tile, one XOR per fetch and a compile-time immediate.
template <int D>
struct FragOffsets {
    int rm0, tr0;
    __device__ __forceinline__ void init(int lane) {
        rm0 = tile_off<D>(lane & 31, lane >> 5);
        const int s = lane & 15;
        const int col = 16 * ((lane >> 4) & 1) + 4 * (s & 3);
        tr0 = tile_off<D>(4 * (lane >> 5) + (s >> 2), col >> 3) + ((col & 4) << 1);
    }
    // tile_off: byte offset of the tile inside `lds` (multiple of 256); rows row0 + l % 32 with
    // row0 a multiple of 16
    __device__ __forceinline__ bf16x8 frag(const char* lds, int tile_off_bytes, int row0, int ks) const {
        const int a = (tile_off_bytes + rm0) ^ (ks << 5);
        return *reinterpret_cast<const bf16x8*>(lds + a + row0 * (D * 2));
    }
    // columns 32 mt + l % 32; rows row16 + 8 (t / 4) + 4h + t % 4 with row16 a multiple of 16
    __device__ __forceinline__ bf16x8 frag_t(const char* lds, int tile_off_bytes, int mt, int row16) const {
        const int a = (tile_off_bytes + tr0) ^ (mt << 6);
        return read_t(lds, a, a ^ 32, row16);
    }
    // Per-fetch address registers for loops whose tile offsets are compile-time constants: with
    //   rm(ks)       = rm0 ^ (ks << 5)              (+ any multiple of 256)
    //   tr(mt, half) = tr0 ^ (mt << 6) ^ (half << 5)
    // kept in registers, a fetch is a register plus an immediate and needs no vector arithmetic.
    __device__ __forceinline__ int rm(int ks) const { return rm0 ^ (ks << 5); }
    __device__ __forceinline__ int tr(int mt, int half) const { return tr0 ^ (mt << 6) ^ (half << 5); }
    static __device__ __forceinline__ bf16x8 read(const char* lds, int rm_ks, int imm) {
        return *reinterpret_cast<const bf16x8*>(lds + rm_ks + imm);
    }
    // imm: tile offset + row16 * row bytes
    static __device__ __forceinline__ bf16x8 read_t(const char* lds, int tr_lo, int tr_hi, int row16, int imm = 0) {
        i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(lds + tr_lo + (imm + row16 * (D * 2))));
        i16x4 hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(lds + tr_hi + (imm + (row16 + 8) * (D * 2))));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        i16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, r);
    }
    // The transposed fetch with the k index in natural order: element t of lane half h <-> row row16 + 8h + t, which
    // pairs with an operand that is read row-major as whole 16-byte chunks.  tr_natural(lane, mt, half) is the
    // address register (half 1 = rows + 4: one step of the row swizzle, 16 bytes), read_t_natural the fetch.
    static __device__ __forceinline__ int tr_natural(int lane, int mt, int half) {
        const int s = lane & 15;
        const int col = 16 * ((lane >> 4) & 1) + 4 * (s & 3);
        const int base = tile_off<D>(8 * (lane >> 5) + (s >> 2), col >> 3) + ((col & 4) << 1);
        return base ^ (mt << 6) ^ (half << 4);
    }
    static __device__ __forceinline__ bf16x8 read_t_natural(const char* lds, int tr_lo, int tr_hi, int row16, int imm = 0) {
        i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(lds + tr_lo + (imm + row16 * (D * 2))));
        i16x4 hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(lds + tr_hi + (imm + (row16 + 4) * (D * 2))));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        i16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, r);
    }
};

// The address registers of all fragments of a [rows x D] tile (static indices only).
template <int D>
struct FragAddrs {
    int rmk[D / 16];
    int trk[D / 32][2];
    __device__ __forceinline__ void init(const FragOffsets<D>& fo) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) rmk[ks] = fo.rm(ks);
#pragma unroll
        for (int mt = 0; mt < D / 32; ++mt) {
            trk[mt][0] = fo.tr(mt, 0);
            trk[mt][1] = fo.tr(mt, 1);
        }
    }
    __device__ __forceinline__ bf16x8 frag(const char* lds, int tile_off_bytes, int row0, int ks) const {
        return FragOffsets<D>::read(lds, rmk[ks], tile_off_bytes + row0 * (D * 2));
    }
    __device__ __forceinline__ bf16x8 frag_t(const char* lds, int tile_off_bytes, int mt, int row16) const {
        return FragOffsets<D>::read_t(lds, trk[mt][0], trk[mt][1], row16, tile_off_bytes);
    }
};

// Operand whose k index runs along the tile's contiguous dimension, but with the k order of
// load_frag_t (element t of half h <-> column 16 ks + 8 (t / 4) + 4h + t % 4), for products
// whose other operand is read transposed.
template <int D>
__device__ __forceinline__ bf16x8 load_frag_perm(const char* tile, int row0, int ks, int lane) {
    const int row = row0 + (lane & 31), h = lane >> 5;
    const u32x2 lo = *reinterpret_cast<const u32x2*>(tile + tile_off<D>(row, 2 * ks) + 8 * h);
    const u32x2 hi = *reinterpret_cast<const u32x2*>(tile + tile_off<D>(row, 2 * ks + 1) + 8 * h);
    u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, r);
}

// Asynchronous copy of a [ROWS x D] bf16 tile from global memory straight into a swizzled LDS
// tile (global_load_lds_dwordx4: no staging registers).  One instruction moves 1 KB per wave and
// lands lane l's 16 bytes at LDS base + 16 l, so the lane that owns LDS position (row, chunk p)
// fetches global chunk p ^ swz(row): the swizzle is applied on the global side.  Rows at or
// beyond rows_valid re-read the last valid row (finite values that the callers mask out).
// The copy is complete for the issuing wave after wait_direct_loads().
template <int D, int ROWS, int NW = 4>  // NW: waves of the workgroup (all of them take part)
__device__ __forceinline__ void load_tile_direct(const __bf16* base, long ld, int row_begin, int rows_valid,
                                                 char* tile, int tid) {
    constexpr int kRowsPerInst = 1024 / (D * 2);
    constexpr int kInst = ROWS / (NW * kRowsPerInst);
    static_assert(ROWS % (NW * kRowsPerInst) == 0, "tile must split evenly over the workgroup's waves");
    const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
    for (int u = 0; u < kInst; ++u) {
        const int row = (u * NW + w) * kRowsPerInst + lane / (D / 8);
        const int c = (lane % (D / 8)) ^ swz<D>(row);
        const int grow = min(row_begin + row, rows_valid - 1);
        // Issued as inline assembly on purpose: for the builtin the compiler cannot tell which LDS
        // bytes a copy in flight will write and drains all of them (s_waitcnt vmcnt(0)) before the
        // next transposing LDS read, i.e. in the middle of the iteration.  Here the wait is ours:
        // wait_direct_loads() right before the barrier that publishes the stage.
        const unsigned dst = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(ATTN_LDS char*)(tile + (u * NW + w) * 1024));
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                     :
                     : "s"(dst), "v"(base + (long)grow * ld + c * 8)
                     : "memory", "m0");
    }
}
__device__ __forceinline__ void wait_direct_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The same copy for the tiles of a streaming loop, with everything that does not change from
// tile to tile taken out of the loop: each lane keeps the byte offset of its 16 bytes relative to
// the tile's first row (one register per copy instruction), the tile's first row is a scalar
// base address, and a copy is one instruction with no vector arithmetic in front of it.
// (Address arithmetic per copy - a 64-bit multiply-add, a clamp, the swizzle - is as expensive
// on the vector unit as the MFMA it feeds.)  Tiles that reach past rows_valid take the
// clamping path of load_tile_direct.  Offsets are 32-bit: ROWS * ld * 2 must stay below 2^32.
template <int D, int ROWS, int NW = 4>
struct TileLoader {
    static constexpr int kRowsPerInst = 1024 / (D * 2);
    static constexpr int kInst = ROWS / (NW * kRowsPerInst);
    static_assert(ROWS % (NW * kRowsPerInst) == 0, "tile must split evenly over the workgroup's waves");
    unsigned voff[kInst];
    unsigned lds0;  // byte offset of this wave's first 1 KB piece inside a tile
    __device__ __forceinline__ void init(int tid, long ld) {
        const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
        for (int u = 0; u < kInst; ++u) {
            const int row = (u * NW + w) * kRowsPerInst + lane / (D / 8);
            const int c = (lane % (D / 8)) ^ swz<D>(row);
            voff[u] = (unsigned)row * (unsigned)ld * 2u + (unsigned)c * 16u;
        }
        lds0 = (unsigned)w * 1024u;
    }
    // The scalar base of the copy instructions: the address is uniform, but the compiler has to
    // be told so where it cannot prove it (it then hands the assembler a vector register pair).
    static __device__ __forceinline__ const __bf16* uniform(const __bf16* ptr) {
        const unsigned long long a = reinterpret_cast<unsigned long long>(ptr);
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
        return reinterpret_cast<const __bf16*>(((unsigned long long)hi << 32) | lo);
    }
    // first_row: address of the tile's first row (uniform); all ROWS rows must exist
    __device__ __forceinline__ void load(const __bf16* first_row_in, char* tile) const {
        const __bf16* first_row = uniform(first_row_in);
        const unsigned t0 =
            __builtin_amdgcn_readfirstlane((unsigned)(size_t)(ATTN_LDS char*)tile) + lds0;
#pragma unroll
        for (int u = 0; u < kInst; ++u) {
            const unsigned dst = t0 + u * NW * 1024;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst), "v"(voff[u]), "s"(first_row)
                         : "memory", "m0");
        }
    }
    // copy instruction u of load() on its own, for callers that spread the copies over their MFMAs
    __device__ __forceinline__ void load_one(int u, const __bf16* first_row_in, char* tile) const {
        const __bf16* first_row = uniform(first_row_in);
        const unsigned dst =
            __builtin_amdgcn_readfirstlane((unsigned)(size_t)(ATTN_LDS char*)tile) + lds0 + u * NW * 1024;
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(dst), "v"(voff[u]), "s"(first_row)
                     : "memory", "m0");
    }
    // any tile: clamps rows at rows_valid - 1 when the tile reaches past the end
    __device__ __forceinline__ void load(const __bf16* base, long ld, int row_begin, int rows_valid, char* tile,
                                         int tid) const {
        if (row_begin + ROWS <= rows_valid)
            load(base + (long)row_begin * ld, tile);
        else
            load_tile_direct<D, ROWS, NW>(base, ld, row_begin, rows_valid, tile, tid);
    }
};

// Marks a register value as used here.  Ordinary global loads issued before the streaming loop
// must be complete before it starts: otherwise the compiler's own wait for them lands inside the
// loop and, vmcnt being one in-order counter, also drains the tile copies in flight.
template <typename T>
__device__ __forceinline__ void settle(const T& v) {
    asm volatile("" : : "v"(v));
}

// Workgroup barrier that orders LDS traffic only: it waits for this wave's LDS operations but
// not for global loads still in flight (__syncthreads would also drain those).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Start row of streamed tile `it` of a workgroup: dense tiles follow one another from t0;
// under a block mask, entry it / sub of the block list picks a 128-row block and it % sub the
// tile inside it.  The list read is forced onto the scalar unit (all values are uniform).
template <int TILE>
__device__ __forceinline__ int tile_start_row(const int32_t* list_idx, int lp0, int t0, int it) {
    constexpr int kSub = 128 / TILE;
    // the result is uniform and is made a scalar here: every address derived from it (tile copies, row
    // statistics) is then scalar arithmetic, not vector instructions that would compete with the MFMAs
    if (list_idx) {
        const int e = __builtin_amdgcn_readfirstlane(lp0 + it / kSub);
        // read through the constant address space: a scalar load (the lists are never written by these kernels),
        // which neither occupies a vector register nor waits behind the tile copies and atomics in flight
        typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
        const const_i32_ptr cidx = (const_i32_ptr)(unsigned long long)list_idx;
        return cidx[e] * 128 + (it % kSub) * TILE;
    }
    return __builtin_amdgcn_readfirstlane((t0 + it) * TILE);
}

// Block lists under the causal rule.  The row list of query block b (ascending key blocks) only
// needs the entries <= b, the column list of key block b (ascending query blocks) only the entries
// >= b: everything else is invisible, and a tile that is not in the list is neither copied nor
// waited for.  All values are uniform (scalar loads).
__device__ __forceinline__ int causal_row_entries(const int32_t* idx, int first, int count, int b) {
    while (count > 0 && idx[first + count - 1] > b) --count;
    return count;
}
__device__ __forceinline__ int causal_col_skip(const int32_t* idx, int first, int count, int b) {
    int skip = 0;
    while (skip < count && idx[first + skip] < b) ++skip;
    return skip;
}

// Head and tile decoding shared by the kernels.  Workgroups are handed to the 8 XCDs round
// robin by linear id, so ids congruent mod 8 share an L2: all tiles of one (batch, head) are
// given to one XCD when the head count allows it.
__device__ __forceinline__ void decode_block(int linear, int tiles, int bh_total, int& bh, int& tile) {
    if ((bh_total & 7) == 0) {
        const int xcd = linear & 7, slot = linear >> 3;
        bh = (slot / tiles) * 8 + xcd;
        tile = slot % tiles;
    } else {
        bh = linear / tiles;
        tile = linear % tiles;
    }
}

// Kernel arguments common to the fused kernels.  Strides are in elements.
struct FusedParams {
    const __bf16 *Q, *K, *V, *O, *dO;
    __bf16 *Oout, *dQ, *dK, *dV;
    const float* LSE;    // [batch*heads, n] natural-log sums (backward input)
    float* LSEout;       // forward output
    float* delta;        // [batch*heads, n] rowsum(dO o O), workspace
    long stride_b, stride_h, stride_n;
    int batch, heads, n;
    float scale;
    int causal;
    // block-sparse lists (nullptr = dense): ptr/idx give, per 128-row block of the resident
    // operand, the 128-row blocks of the streamed operand that are visible, ascending.
    const int32_t *list_ptr, *list_idx;
    // under a block mask, optionally: the 128-row blocks of the resident operand in the order the
    // workgroups take them (longest list first), nullptr = ascending
    const int32_t* order;
    // masks per (batch, head): entries between the list_ptr (order) arrays of consecutive pairs; 0 = one shared mask
    int list_stride, order_stride;
};

}  // namespace attn
