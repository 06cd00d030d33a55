// Device-side building blocks shared by the forward and backward kernels (gfx950 only).
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (D = A * B + C, A is 32 x 16, B is 16 x 32), lane l:
//   A operand: row  l % 32, k = 8 * (l / 32) .. + 7          (8 bf16 in 4 VGPRs)
//   B operand: col  l % 32, k = 8 * (l / 32) .. + 7
//   C / D    : col  l % 32, register i holds row 8 * (i / 4) + 4 * (l / 32) + i % 4   (16 fp32)
// Every kernel here computes transposed products (keys or head-dim along the rows, the wave's
// own 32 queries -- or keys, in the dK/dV pass -- along the columns), so that
//   * one lane owns one query (key): row max / row sum are in-lane reductions plus ONE exchange
//     with lane l ^ 32, and the per-row scalars (max, sum, LSE, D) are plain lane scalars;
//   * an accumulator fragment, converted to bf16, is directly the B operand of the next
//     product: registers 8t .. 8t+7 of a block hold the k-slice {16t + 8*(ii/4) + 4*(l/32) + ii%4}.
//     A contraction does not care about the order of k as long as A uses the same order, so the
//     A operand of that product is fetched with the matching permutation.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/hspmd_attn.h"
#include <stdint.h>

namespace hspmd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kThreads = 256;   // 4 waves of 64
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- LDS tiles --------------------------------------------------------------------------
// A tile is ROWS x D bf16, row pitch D*2 bytes, no padding.  16-byte chunks of a row are
// XOR-swizzled with a function of the row so that both access patterns below are free of
// bank conflicts (64 banks x 4 B):
//   * 16 lanes reading the same logical chunk of 16 consecutive rows (MFMA operand whose k
//     runs along the row), and
//   * the transpose read, where a 32-lane half reads 64 contiguous bytes of each of 4
//     consecutive rows (MFMA operand whose k runs down the rows).
template <int D>
__device__ __forceinline__ int swizzle(int row, int chunk) {
    if constexpr (D == 128) {
        return chunk ^ (((row & 3) << 2) | ((row >> 2) & 3));
    } else {
        return chunk ^ ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    }
}

// byte offset of element (row, col) inside a tile; col is a multiple of 4
template <int D>
__device__ __forceinline__ int tile_offset(int row, int col) {
    return row * (D * 2) + (swizzle<D>(row, col >> 3) << 4) + ((col & 7) << 1);
}

// One wave-wide global -> LDS copy of SIZE bytes per lane (global_load_lds_dword / _dwordx4): lane i's
// data lands at lds_dst + SIZE * i.  Written as inline assembly on purpose: when the compiler knows that
// such copies are in flight it makes every later LDS transpose read wait for all of them (vmcnt(0)),
// which serialises the prefetch.  Here the copies are ordered by hand instead: the issuing wave waits
// with wait_tile_loads*() before the workgroup barrier that publishes the tile.  "memory" keeps the
// compiler from moving LDS accesses across the issue point.  M0 (the LDS base of the copy) is written
// inside the statement; nothing else in these kernels keeps a value in M0 (the compiler sets it up
// immediately before each of its own uses), and it is a reserved register that cannot be named as a clobber.
// LDS destinations are passed as 32-bit LDS byte addresses (lds_address of the kernel's shared array plus
// an offset): a generic pointer would be converted, null check included, at every copy.
__device__ __forceinline__ uint32_t lds_address(const void* shared_ptr) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)shared_ptr;
}

template <int SIZE>
__device__ __forceinline__ void global_to_lds(const void* src, uint32_t lds_dst) {
    static_assert(SIZE == 4 || SIZE == 16, "dword or dwordx4");
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_dst);
    if constexpr (SIZE == 16) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                     :: "s"(m0), "v"(src) : "memory");
    } else {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                     :: "s"(m0), "v"(src) : "memory");
    }
}

// Same copy with the global address given as a wave-uniform base plus a per-lane unsigned byte offset
// (the saddr form): the per-lane offsets of a tile are loop-invariant, so issuing a tile costs no VALU work.
template <int SIZE>
__device__ __forceinline__ void global_to_lds(const void* uniform_base, uint32_t lane_byte_offset, uint32_t lds_dst) {
    static_assert(SIZE == 4 || SIZE == 16, "dword or dwordx4");
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_dst);
    // readfirstlane returns a signed int: widen each half as unsigned, or a low half with bit 31 set
    // would sign-extend over the high half and produce a wild address
    const uint64_t b = (uint64_t)(uintptr_t)uniform_base;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
    const uint64_t base = ((uint64_t)hi << 32) | (uint64_t)lo;
    if constexpr (SIZE == 16) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(m0), "v"(lane_byte_offset), "s"(base) : "memory");
    } else {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                     :: "s"(m0), "v"(lane_byte_offset), "s"(base) : "memory");
    }
}

// Global -> LDS copy of a ROWS x D tile without a trip through registers.
// One wave instruction moves 64 x 16 B into 1024 consecutive LDS bytes (lane i lands at base + 16 i),
// so the swizzle is applied on the global side: the lane that owns physical chunk p of row r
// fetches logical chunk p ^ f(r).  Rows at or beyond seq_len are replaced by the last valid row:
// they only ever meet a zero weight, and a finite duplicate keeps 0 * x = 0.
// The copies are asynchronous: wait_tile_loads() + a workgroup barrier make them visible.
template <int D, int ROWS>
struct TileCopy {
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kRowsPerInstr = 64 / kChunksPerRow;
    static constexpr int kInstr = ROWS / kRowsPerInstr;
    static constexpr int kPerWave = kInstr / 4;
    static_assert(kInstr % 4 == 0, "tile must divide over 4 waves");
    uint32_t off[kPerWave];   // byte offset of this lane's chunk from the tile's first row, per instruction
    int chunk_bytes;          // swizzled column offset (bytes) of this lane's chunk: same for every instruction
    int row_in_instr;
    int last_chunk;           // head_dim / 8 - 1: the row's last chunk that exists in memory

    // stride: token stride of the tensor in elements (loop-invariant).  head_dim (elements per row in memory) may
    // be smaller than the tile width D: the pad chunks of an LDS row then repeat the row's last valid chunk, so
    // that they hold finite values (they only ever meet zeros of the other operand, or produce columns nobody stores)
    __device__ __forceinline__ void init(int64_t stride, int wave, int lane, int head_dim = D) {
        row_in_instr = lane / kChunksPerRow;
        last_chunk = head_dim / 8 - 1;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int r = (i * 4 + wave) * kRowsPerInstr + row_in_instr;
            const int c = min(swizzle<D>(r, lane % kChunksPerRow), last_chunk);
            off[i] = (uint32_t)(r * (int)stride + c * 8) * 2u;
        }
    }
    // instruction I (of kPerWave) of a whole-tile copy; first_row points at the tile's first row, column 0
    template <int I>
    __device__ __forceinline__ void issue_full_one(uint32_t tile, const uint16_t* first_row, int wave) const {
        static_assert(I >= 0 && I < kPerWave, "instruction index");
        global_to_lds<16>(first_row, off[I], tile + (I * 4 + wave) * 1024);
    }
    // the same with the index as a (compile-time constant after unrolling) argument
    __device__ __forceinline__ void issue_full_one_at(int i, uint32_t tile, const uint16_t* first_row, int wave) const {
        global_to_lds<16>(first_row, off[i], tile + (i * 4 + wave) * 1024);
    }
    // whole tile inside the sequence: rows row0 .. row0+ROWS-1 all exist.  slab points at row 0, column 0.
    __device__ __forceinline__ void issue_full(uint32_t tile, const uint16_t* slab, int64_t stride, int row0, int wave) const {
        const uint16_t* base = slab + (int64_t)row0 * stride;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) global_to_lds<16>(base, off[i], tile + (i * 4 + wave) * 1024);
    }
    // tile that runs past the end of the sequence: per-lane row clamp
    __device__ __forceinline__ void issue_clamped(uint32_t tile, const uint16_t* slab, int64_t stride, int row0, int seq_len,
                                                  int wave, int lane) const {
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int blk = i * 4 + wave;
            const int r = blk * kRowsPerInstr + row_in_instr;
            const int c = min(swizzle<D>(r, lane % kChunksPerRow), last_chunk);
            const int row = min(row0 + r, seq_len - 1);
            global_to_lds<16>(slab + (int64_t)row * stride + c * 8, tile + blk * 1024);
        }
    }
    __device__ __forceinline__ void issue(uint32_t tile, const uint16_t* slab, int64_t stride, int row0, int seq_len,
                                          int wave, int lane) const {
        if (row0 + ROWS <= seq_len) issue_full(tile, slab, stride, row0, wave);
        else issue_clamped(tile, slab, stride, row0, seq_len, wave, lane);
    }
};

// all of this wave's outstanding global loads (direct-to-LDS copies included) have landed
__device__ __forceinline__ void wait_tile_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// all but the newest N (N < 16) of this wave's global loads have landed (loads complete in order)
template <int N>
__device__ __forceinline__ void wait_tile_loads_except() {
    static_assert(N >= 0 && N < 16, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// A operand whose k runs along the tile's rows' columns: 8 consecutive elements of one row.
//   rows: 32-row block `rb`; k-step kk covers columns 16*kk .. 16*kk+15
template <int D>
__device__ __forceinline__ bf16x8 read_rowmajor_frag(const char* tile, int rb, int kk, int lane) {
    const int row = rb * 32 + (lane & 31);
    return *reinterpret_cast<const bf16x8*>(tile + tile_offset<D>(row, kk * 16 + ((lane >> 5) << 3)));
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane 4*i + c supplies the address of 4
// consecutive 16-bit elements (row i, columns 4c .. 4c+3 of a 4 x 16 block); lane n of the group
// receives column n of that block, i.e. elements (0,n), (1,n), (2,n), (3,n).
__device__ __forceinline__ s16x4 lds_transpose_read(const char* p) {
    // a plain address-space cast (no trip through an integer) keeps the pointer's provenance, so the compiler
    // can tell these reads from the in-flight global->LDS copies and does not wait for those first
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(const_cast<char*>(p)));
}

// A operand whose k runs DOWN the tile's rows (the tile is used transposed):
//   result row (MFMA M index) = column 32*cb + lane%32 of the tile,
//   k = the 16 tile rows 16*t .. 16*t+15 in the order of an accumulator fragment
//       (lane half hh gets rows 16t + 4hh + {0..3} and 16t + 8 + 4hh + {0..3}).
template <int D>
__device__ __forceinline__ bf16x8 read_transposed_frag(const char* tile, int cb, int t, int lane) {
    const int c16 = lane & 15;
    const int col = cb * 32 + (((lane >> 4) & 1) << 4) + ((c16 & 3) << 2);
    const int row = t * 16 + ((lane >> 5) << 2) + (c16 >> 2);
    const s16x4 lo = lds_transpose_read(tile + tile_offset<D>(row, col));
    const s16x4 hi = lds_transpose_read(tile + tile_offset<D>(row + 8, col));
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = lo;
    u.s.b = hi;
    return u.v;
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// value held by lane l ^ 32 (the lane that owns the other half of this lane's column)
__device__ __forceinline__ float partner32(float x) { return __shfl_xor(x, 32, 64); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 p = {(__bf16)lo, (__bf16)hi};
    return *reinterpret_cast<uint32_t*>(&p);
}

// registers 8*tt .. 8*tt+7 of an accumulator block as a bf16 B operand
__device__ __forceinline__ bf16x8 frag_to_bf16(const f32x16& c, int tt) {
    union { u32x4 u; bf16x8 v; } r;
    r.u[0] = pack_bf16(c[8 * tt + 0], c[8 * tt + 1]);
    r.u[1] = pack_bf16(c[8 * tt + 2], c[8 * tt + 3]);
    r.u[2] = pack_bf16(c[8 * tt + 4], c[8 * tt + 5]);
    r.u[3] = pack_bf16(c[8 * tt + 6], c[8 * tt + 7]);
    return r.v;
}

// row (MFMA M index within a 32-block) held in accumulator register i by this lane
__device__ __forceinline__ int acc_row(int i, int lane) { return ((i >> 2) << 3) + ((lane >> 5) << 2) + (i & 3); }

// writes 4 consecutive gradient elements of one row (bf16 or fp32)
__device__ __forceinline__ void store_grad4(void* base, int64_t elem, bool f32, float a, float b, float c, float d) {
    if (f32) {
        *reinterpret_cast<f32x4*>(static_cast<float*>(base) + elem) = f32x4{a, b, c, d};
    } else {
        u32x2 w;
        w[0] = pack_bf16(a, b);
        w[1] = pack_bf16(c, d);
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(base) + elem) = w;
    }
}

// Coalesced store of a wave's 32 x D result tile.  The transposed products leave one ROW per lane pair (lane
// l and l + 32 hold row l % 32: register 4 i4 + j of fragment db is column 32 db + 8 i4 + 4 (l / 32) + j), so a
// direct store writes 64 scattered 8- or 16-byte pieces per instruction, one partial line each.  The tile goes
// through a wave-private LDS area instead (32 rows of D elements, 16-byte chunks XOR-swizzled by the row so that
// writes and reads are conflict-free) and every store instruction then writes whole rows.  The caller makes sure
// no wave still reads the LDS area (a workgroup barrier after the last tile); the area itself is private to the
// wave, and LDS accesses of one wave complete in order, so no barrier is needed between its writes and reads.
//   valid_rows: rows 0 .. valid_rows-1 exist; head_dim: columns that exist in memory (<= D, a multiple of 8)
//   ACCUM: add to what the destination holds (fp32 only)
// FULL: all 32 rows and all D columns exist (decided per wave by the callers below).  Without the per-row test the
// second loop is straight-line code: the LDS reads are issued together and the stores follow as the data arrives,
// instead of one LDS round trip per store.
template <int D, bool ACCUM, bool FULL>
__device__ __forceinline__ void store_tile_f32_rows(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, float* first_row,
                                                    int64_t row_stride, int valid_rows, int head_dim, int lane) {
    constexpr int kChunks = D / 4;                // 16-byte chunks per row
    const int r = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const int chunk = (db * 32 + i4 * 8 + hh * 4) / 4;
            *reinterpret_cast<f32x4*>(wave_lds + (r * kChunks + (chunk ^ (r & (kChunks - 1)))) * 16) =
                f32x4{acc[db][4 * i4 + 0] * mul, acc[db][4 * i4 + 1] * mul, acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul};
        }
    constexpr int kRowsPerInstr = 64 / kChunks;
    const int chunk = lane % kChunks;
    float* const lane_dst = first_row + (lane / kChunks) * row_stride + chunk * 4;   // this lane's piece of rows 0 .. kRowsPerInstr-1
#pragma unroll
    for (int it = 0; it < 32 / kRowsPerInstr; ++it) {
        const int row = it * kRowsPerInstr + lane / kChunks;
        if (FULL || (row < valid_rows && chunk * 4 < head_dim)) {
            f32x4 v = *reinterpret_cast<const f32x4*>(wave_lds + (row * kChunks + (chunk ^ (row & (kChunks - 1)))) * 16);
            f32x4* dst = reinterpret_cast<f32x4*>(lane_dst + it * kRowsPerInstr * row_stride);
            if constexpr (ACCUM) {
                const f32x4 old = *dst;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] += old[j];
            }
            *dst = v;
        }
    }
}

template <int D, bool ACCUM>
__device__ __forceinline__ void store_tile_f32(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, float* first_row,
                                               int64_t row_stride, int valid_rows, int head_dim, int lane) {
    if (valid_rows >= 32 && head_dim == D)
        store_tile_f32_rows<D, ACCUM, true>(wave_lds, acc, mul, first_row, row_stride, valid_rows, head_dim, lane);
    else
        store_tile_f32_rows<D, ACCUM, false>(wave_lds, acc, mul, first_row, row_stride, valid_rows, head_dim, lane);
}

// The same for a bf16 destination: rows of D bf16 in LDS (8-byte pieces in, 16-byte chunks out).
template <int D, bool FULL>
__device__ __forceinline__ void store_tile_bf16_rows(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, uint16_t* first_row,
                                                     int64_t row_stride, int valid_rows, int head_dim, int lane) {
    constexpr int kChunks = D / 8;                // 16-byte chunks (8 bf16) per row
    const int r = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const int col = db * 32 + i4 * 8 + hh * 4;           // 4 elements = half a chunk
            u32x2 w;
            w[0] = pack_bf16(acc[db][4 * i4 + 0] * mul, acc[db][4 * i4 + 1] * mul);
            w[1] = pack_bf16(acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul);
            *reinterpret_cast<u32x2*>(wave_lds + (r * kChunks + ((col / 8) ^ (r & (kChunks - 1)))) * 16 + (col & 4) * 2) = w;
        }
    constexpr int kRowsPerInstr = 64 / kChunks;
    const int chunk = lane % kChunks;
    uint16_t* const lane_dst = first_row + (lane / kChunks) * row_stride + chunk * 8;
#pragma unroll
    for (int it = 0; it < 32 / kRowsPerInstr; ++it) {
        const int row = it * kRowsPerInstr + lane / kChunks;
        if (FULL || (row < valid_rows && chunk * 8 < head_dim))
            *reinterpret_cast<u32x4*>(lane_dst + it * kRowsPerInstr * row_stride) =
                *reinterpret_cast<const u32x4*>(wave_lds + (row * kChunks + (chunk ^ (row & (kChunks - 1)))) * 16);
    }
}

template <int D>
__device__ __forceinline__ void store_tile_bf16(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, uint16_t* first_row,
                                                int64_t row_stride, int valid_rows, int head_dim, int lane) {
    if (valid_rows >= 32 && head_dim == D)
        store_tile_bf16_rows<D, true>(wave_lds, acc, mul, first_row, row_stride, valid_rows, head_dim, lane);
    else
        store_tile_bf16_rows<D, false>(wave_lds, acc, mul, first_row, row_stride, valid_rows, head_dim, lane);
}

// The same with the transposed rotary-embedding rotation applied on the way out (the gradient with respect to the
// unrotated vector, given the gradient with respect to the rotated one).  RoPE pairs column i with column
// i + head_dim/2 and turns the pair of a token at position p by p * theta_i (model configuration table of the paper:
// position encoding RoPE; rotate-half pairing); the transposed map turns it back:
//   x_lo = y_lo cos + y_hi sin,   x_hi = y_hi cos - y_lo sin.
// The tile is staged as fp32 whatever the destination type; a lane then fetches 4 columns of the low half and their
// 4 partner columns (head_dim/2 is a multiple of 4) from LDS and writes both; cos and sin come from the caller's table
// [position][head_dim/2] of (cos, sin) pairs, `table_row0` pointing at the position of the tile's first row
// (the 32 rows are consecutive positions).
//   ACCUM: add to what the destination holds (fp32 only; the rotation is linear, so a sum of rotated shares is the
//   rotated sum)
//   FULL: all 32 rows and all D columns exist (straight-line code, see store_tile_f32_rows)
template <int D, bool ACCUM, bool FULL>
__device__ __forceinline__ void store_tile_rope_transposed_rows(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, void* base,
                                                                int64_t first_elem, bool f32, int64_t row_stride, int valid_rows,
                                                                int head_dim, const float* table_row0, int lane) {
    constexpr int kChunks = D / 4;             // 16-byte chunks per staged row
    constexpr int kPairs = D / 8;              // lanes per row: lane c owns chunk c of the low half and its partner
    constexpr int kRowsPerInstr = 64 / kPairs;
    constexpr int kIters = 32 / kRowsPerInstr;
    const int half_chunks = head_dim / 8;
    const int c = lane % kPairs, sub_row = lane / kPairs;
    // all table reads first, so that their latency is paid once and overlaps the staging
    f32x4 t01[kIters], t23[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int row = it * kRowsPerInstr + sub_row;
        if (FULL || (row < valid_rows && c < half_chunks)) {
            const float* t = table_row0 + ((int64_t)row * (head_dim / 2) + c * 4) * 2;
            t01[it] = *reinterpret_cast<const f32x4*>(t);
            t23[it] = *reinterpret_cast<const f32x4*>(t + 4);
        }
    }
    const int r = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const int chunk = (db * 32 + i4 * 8 + hh * 4) / 4;
            *reinterpret_cast<f32x4*>(wave_lds + (r * kChunks + (chunk ^ (r & (kChunks - 1)))) * 16) =
                f32x4{acc[db][4 * i4 + 0] * mul, acc[db][4 * i4 + 1] * mul, acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul};
        }
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int row = it * kRowsPerInstr + sub_row;
        if (FULL || (row < valid_rows && c < half_chunks)) {
            const int sw = row & (kChunks - 1);
            const f32x4 lo = *reinterpret_cast<const f32x4*>(wave_lds + (row * kChunks + (c ^ sw)) * 16);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(wave_lds + (row * kChunks + ((c + half_chunks) ^ sw)) * 16);
            const float cs[4] = {t01[it][0], t01[it][2], t23[it][0], t23[it][2]};
            const float sn[4] = {t01[it][1], t01[it][3], t23[it][1], t23[it][3]};
            const int64_t e = first_elem + row * row_stride + c * 4;
            f32x4 x_lo, x_hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x_lo[j] = lo[j] * cs[j] + hi[j] * sn[j];
                x_hi[j] = hi[j] * cs[j] - lo[j] * sn[j];
            }
            if constexpr (ACCUM) {
                float* dst = static_cast<float*>(base) + e;
                const f32x4 old_lo = *reinterpret_cast<const f32x4*>(dst);
                const f32x4 old_hi = *reinterpret_cast<const f32x4*>(dst + head_dim / 2);
#pragma unroll
                for (int j = 0; j < 4; ++j) { x_lo[j] += old_lo[j]; x_hi[j] += old_hi[j]; }
            }
            store_grad4(base, e, f32, x_lo[0], x_lo[1], x_lo[2], x_lo[3]);
            store_grad4(base, e + head_dim / 2, f32, x_hi[0], x_hi[1], x_hi[2], x_hi[3]);
        }
    }
}

template <int D, bool ACCUM = false>
__device__ __forceinline__ void store_tile_rope_transposed(char* wave_lds, const f32x16 (&acc)[D / 32], float mul, void* base,
                                                           int64_t first_elem, bool f32, int64_t row_stride, int valid_rows,
                                                           int head_dim, const float* table_row0, int lane) {
    if (valid_rows >= 32 && head_dim == D)
        store_tile_rope_transposed_rows<D, ACCUM, true>(wave_lds, acc, mul, base, first_elem, f32, row_stride, valid_rows, head_dim,
                                                        table_row0, lane);
    else
        store_tile_rope_transposed_rows<D, ACCUM, false>(wave_lds, acc, mul, base, first_elem, f32, row_stride, valid_rows, head_dim,
                                                         table_row0, lane);
}

// Scheduling hint for one basic block: N times {1 MFMA, DS LDS reads, VA VALU instructions}, in that
// order, as one pipeline with the given id (llvm.amdgcn.sched.group.barrier; arguments must be constants).
// VMASK selects what counts as a VALU instruction: 0x002 plain VALU, 0x402 plain VALU and transcendentals
// (v_exp_f32 belongs to a class of its own and is left out of a 0x002 group).
template <int N, int DS, int VA, int ID, int VMASK = 0x002>
struct InterleaveHint {
    static __device__ __forceinline__ void apply() {
        if constexpr (N > 0) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, ID);
            if constexpr (DS > 0) __builtin_amdgcn_sched_group_barrier(0x100, DS, ID);
            if constexpr (VA > 0) __builtin_amdgcn_sched_group_barrier(VMASK, VA, ID);
            InterleaveHint<N - 1, DS, VA, ID, VMASK>::apply();
        }
    }
};

// Geometry of one work item.  The packed self-attention lists carry (token_start, seq_len); the block variant
// carries separate query and key chunks and the shift of the causal mask.  With BLOCK = false the chunk fields
// are copies and offset is the constant 0, so the general index arithmetic folds back to the plain one.
struct ItemGeom {
    int q_start, q_len, k_start, k_len, offset, tile, head;
    int q_pos;   // position of the chunk's first row inside its sequence (0 when !BLOCK); the key chunk's is q_pos - offset
};
template <bool BLOCK>
__device__ __forceinline__ ItemGeom load_item(const hspmd_work_item* items, const hspmd_block_item* block_items, int idx) {
    if constexpr (BLOCK) {
        const hspmd_block_item it = block_items[idx];
        return ItemGeom{it.q_start, it.q_len, it.k_start, it.k_len, it.offset, it.tile, it.head, it.q_pos};
    } else {
        const hspmd_work_item it = items[idx];
        return ItemGeom{it.token_start, it.seq_len, it.token_start, it.seq_len, 0, it.tile, it.head, 0};
    }
}

// Work distribution of the persistent kernels.  A launch starts as many workgroups as the device holds at once;
// workgroup b begins with slot b of the launch-ordered list (slot p belongs to queue p % kQueues, and workgroups are
// handed to the XCDs round-robin, so queue q is served by the workgroups of XCD q) and then draws further slots of
// ITS OWN queue from a counter in device memory, in list order: the same order in which the hardware would have
// dispatched one workgroup per slot, without the time a compute unit spends between two workgroups (several
// microseconds per item, a fifth of the time on packs of short sequences).  Which workgroup computes an item never
// changes the item's result.
//   counters[0 .. kQueues-1]: draws made from each queue; counters[kQueues]: workgroups that have left.
// The last workgroup to leave puts all of them back to zero, so the next launch that uses the same counters (it must
// be ordered after this one on the device) starts from a clean state and nothing on the host has to reset them.
constexpr int kQueues = 8;          // = kNumXcd of the scheduler
constexpr int kQueueInts = 16;      // int32 per counter block (kQueues + 1 used)
struct ItemQueue {
    int32_t* counters;
    int queue, first_round;
    __device__ __forceinline__ void init(int32_t* c) {
        counters = c;
        queue = blockIdx.x % kQueues;
        first_round = gridDim.x / kQueues;     // the grid is a multiple of kQueues: slots 0 .. gridDim.x-1 are taken
    }
    // one thread per workgroup: the list index of the workgroup's next item (past the end when the queue is empty)
    __device__ __forceinline__ int draw() const {
        const int k = __hip_atomic_fetch_add(counters + queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return (first_round + k) * kQueues + queue;
    }
    // one thread per workgroup, after its last draw
    __device__ __forceinline__ void leave() const {
        const int gone = __hip_atomic_fetch_add(counters + kQueues, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if (gone == (int)gridDim.x - 1) {
#pragma unroll
            for (int i = 0; i <= kQueues; ++i)
                __hip_atomic_store(counters + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace hspmd
