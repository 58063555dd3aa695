// Shared host/device helpers of libwindq (gfx950 only).
//
// Kernel-wide design: a weight matrix is cut into tiles of TILE_ROWS rows x one chunk
// (chunk_w columns).  A workgroup loads its tile from HBM with coalesced 128-bit loads
// and stages it in LDS in the input's own element type; then every lane owns ONE group
// (one row of the tile) and walks along its chunk_w columns.  A group's min, max, mean|w|
// and all of its quantizer parameters are therefore private to a lane: no cross-lane
// traffic and no redundant parameter arithmetic inside the hot loops.  Lanes are combined
// only once per tile, in a fixed order, so every result is bit-reproducible.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "windq.h"

namespace windq {

constexpr int TILE_ROWS = 64;   // rows per tile = lanes per wavefront

// Geometry of the unit decomposition of one matrix (Sec. 3.1: column-chunk units).
struct Geometry {
    int64_t rows, cols, ld;
    int32_t chunk_w;
    int64_t R_u;             // rows per unit
    int64_t n_chunks;        // cols / chunk_w
    int64_t n_rb;            // row blocks = rows / R_u
    int64_t U;               // units = n_rb * n_chunks
    int64_t tiles_per_unit;  // ceil(R_u / TILE_ROWS)
    int64_t n_tiles;         // U * tiles_per_unit
};

int check_matrix(const windq_mat* M);
int make_geometry(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, Geometry* g);
int check_clip_grid(const float* clip_grid, int32_t K);
bool aligned(const void* p, size_t a);
size_t round_up(size_t x, size_t a);

// Clip grid handed to kernels by value (lands in the kernarg segment, read with
// scalar loads).
struct ClipGrid {
    float p[WINDQ_MAX_CLIP];
};

// LDS bytes of a raw tile: row stride = row bytes + 16.  With a stride of 4*odd dwords the
// 64 lanes' 128-bit reads of 64 different rows spread evenly over the LDS banks.
inline size_t raw_tile_lds_bytes(int32_t dtype, int32_t chunk_w) {
    return (size_t)TILE_ROWS * ((size_t)chunk_w * (dtype == WINDQ_BF16 ? 2 : 4) + 16);
}

// Row stride of a tile's protection-mask bytes staged in LDS: an odd number of dwords where
// the width allows, so that 64 lanes reading 64 rows spread over the banks.
__host__ __device__ inline int32_t mask_row_stride(int32_t chunk_w) { return (((chunk_w >> 3) + 3) & ~3) + 4; }
inline size_t mask_tile_lds_bytes(int32_t chunk_w) { return (size_t)TILE_ROWS * (size_t)mask_row_stride(chunk_w); }

// Raises the dynamic-LDS limit of a kernel when a tile needs more than the 64 KB a
// workgroup gets by default (gfx950 has 160 KB per CU).
int ensure_lds(const void* kernel, size_t bytes);

#ifdef __HIPCC__

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Decode tile index -> (unit, first row, valid rows, first column).
struct TileCoord {
    int64_t u;        // unit index
    int64_t row0;     // first matrix row of the tile
    int64_t lrow0;    // first row of the tile, local to the unit
    int32_t nrows;    // valid rows in the tile (1..TILE_ROWS)
    int64_t col0;     // first column of the chunk
    int64_t t;        // tile index inside the unit
};

// Tiles are numbered so that consecutive workgroups walk across the chunks of one band
// of rows: a band of 64 rows is contiguous in HBM row by row, and neighbouring
// workgroups (which land on different XCDs round-robin) share DRAM pages, not L2 lines.
// (A matrix has fewer than 2^31 tiles, checked on the host: the two divisions are 32-bit ones.)
__device__ __forceinline__ TileCoord tile_coord(const Geometry& g, int64_t tile) {
    TileCoord tc;
    const uint32_t nc = (uint32_t)g.n_chunks, tpu = (uint32_t)g.tiles_per_unit;
    const uint32_t band32 = (uint32_t)tile / nc;     // band = rb * tiles_per_unit + t
    const int64_t j = (int64_t)((uint32_t)tile - band32 * nc);
    const uint32_t rb32 = band32 / tpu;
    const int64_t rb = (int64_t)rb32;
    tc.t = (int64_t)(band32 - rb32 * tpu);
    tc.u = rb * g.n_chunks + j;
    tc.lrow0 = tc.t * TILE_ROWS;
    tc.row0 = rb * g.R_u + tc.lrow0;
    const int64_t left = g.R_u - tc.lrow0;
    tc.nrows = left < TILE_ROWS ? (int32_t)left : TILE_ROWS;
    tc.col0 = j * g.chunk_w;
    return tc;
}

// Tile t of unit u.
__device__ __forceinline__ TileCoord tile_coord_of_unit(const Geometry& g, int64_t u, int64_t t) {
    TileCoord tc;
    const int64_t rb = (int64_t)((uint32_t)u / (uint32_t)g.n_chunks);
    const int64_t j = u - rb * g.n_chunks;
    tc.t = t;
    tc.u = u;
    tc.lrow0 = t * TILE_ROWS;
    tc.row0 = rb * g.R_u + tc.lrow0;
    const int64_t left = g.R_u - tc.lrow0;
    tc.nrows = left < TILE_ROWS ? (int32_t)left : TILE_ROWS;
    tc.col0 = j * g.chunk_w;
    return tc;
}

template <int DT>
struct Elem {
    static constexpr int bytes = DT == WINDQ_BF16 ? 2 : 4;
};

// The pieces first, first + stride, first + 2 stride, ... of a tile whose rows hold `pieces` pieces each:
// row and piece in the row by stepping (one division at the start instead of one per piece).
struct PieceWalk {
    int32_t r, pc;                  // row of the tile, piece in the row
    int32_t dr, dpc, pieces;
    __device__ __forceinline__ PieceWalk(int32_t first, int32_t stride, int32_t pieces_per_row) : pieces(pieces_per_row) {
        r = (int32_t)((uint32_t)first / (uint32_t)pieces);
        pc = first - r * pieces;
        dr = (int32_t)((uint32_t)stride / (uint32_t)pieces);
        dpc = stride - dr * pieces;
    }
    __device__ __forceinline__ void next() {
        r += dr;
        pc += dpc;
        if (pc >= pieces) {
            pc -= pieces;
            ++r;
        }
    }
};

// Cooperative load of one tile into LDS, element type unchanged.  Each thread moves 16
// bytes per step; 16 (bf16, chunk 128) neighbouring threads cover one contiguous row
// segment.  Rows past the end of the unit are filled with zeros.
// NB pieces per thread and step have their loads issued together before any is stored: with
// one wavefront per tile (16 steps at bf16, chunk 128) that is 4 memory latencies instead of 16.
template <int DT, int NB = 4>
__device__ __forceinline__ void load_tile_raw(const void* __restrict__ data, int64_t ld, const TileCoord& tc,
                                              int32_t chunk_w, char* __restrict__ tile) {
    constexpr int EB = Elem<DT>::bytes;
    const uint32_t pieces = (uint32_t)(chunk_w * EB) >> 4;   // 16-byte pieces per row
    const int32_t row_bytes = chunk_w * EB + 16;
    const int32_t total = TILE_ROWS * (int32_t)pieces;
    const uint32_t nthreads = blockDim.x;
    // A thread's pieces lie nthreads apart: (row, piece) of the first by one division, of the others
    // by stepping (dr rows and dpc pieces further, one more row when the piece index wraps).
    uint32_t r = threadIdx.x / pieces;
    uint32_t pc = threadIdx.x - r * pieces;
    const uint32_t dr = nthreads / pieces, dpc = nthreads - dr * pieces;          // wave-uniform
    const int64_t row_step = ld * EB;
    const int64_t src_step = (int64_t)dr * row_step + (int64_t)dpc * 16;
    const int64_t src_wrap = row_step - (int64_t)pieces * 16;
    const int32_t dst_step = (int32_t)dr * row_bytes + (int32_t)dpc * 16;
    const int32_t dst_wrap = row_bytes - (int32_t)pieces * 16;
    const char* __restrict__ src = static_cast<const char*>(data) + ((tc.row0 + (int64_t)r) * ld + tc.col0) * EB + (int64_t)pc * 16;
    int32_t dst = (int32_t)r * row_bytes + (int32_t)pc * 16;
    for (int32_t i0 = threadIdx.x; i0 < total; i0 += NB * (int32_t)nthreads) {
        uint4 v[NB];
        int32_t at[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int32_t i = i0 + k * (int32_t)nthreads;
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            at[k] = dst;
            if (i < total && (int32_t)r < tc.nrows) v[k] = *reinterpret_cast<const uint4*>(src);
            r += dr;
            pc += dpc;
            src += src_step;
            dst += dst_step;
            if (pc >= pieces) {
                pc -= pieces;
                r += 1u;
                src += src_wrap;
                dst += dst_wrap;
            }
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            if (i0 + k * (int32_t)nthreads < total) *reinterpret_cast<uint4*>(tile + at[k]) = v[k];
        }
    }
}

// Cooperative load of a tile's mask bytes (one per 8 columns and row) into LDS, rows past the
// unit's end as zeros.  Kernels that give a lane a row read them from there: a byte load from
// global memory inside a lane's column loop would put a memory latency into every step.
__device__ __forceinline__ void load_mask_tile(const uint8_t* __restrict__ mask, int64_t mask_ld, const TileCoord& tc,
                                               int32_t chunk_w, uint8_t* __restrict__ mtile) {
    const int32_t mb = chunk_w >> 3;                 // mask bytes per row of the tile
    const int32_t mstride = mask_row_stride(chunk_w);
    const uint8_t* __restrict__ src = mask + tc.row0 * mask_ld + (tc.col0 >> 3);
    const bool by16 = (mb & 15) == 0 && (mask_ld & 15) == 0 && (reinterpret_cast<uintptr_t>(src) & 15) == 0;
    const bool by4 = (mb & 3) == 0 && (mask_ld & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 3) == 0;
    if (by16) {                                      // e.g. chunk 128: one 16-byte load per row
        const int32_t pieces = mb >> 4;
        for (int32_t i = threadIdx.x; i < TILE_ROWS * pieces; i += blockDim.x) {
            const int32_t r = i / pieces, pc = i - r * pieces;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (r < tc.nrows) v = *reinterpret_cast<const uint4*>(src + r * mask_ld + pc * 16);
            uint32_t* dst = reinterpret_cast<uint32_t*>(mtile + r * mstride + pc * 16);
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
    } else if (by4) {
        const int32_t pieces = mb >> 2;
        for (int32_t i = threadIdx.x; i < TILE_ROWS * pieces; i += blockDim.x) {
            const int32_t r = i / pieces, pc = i - r * pieces;
            uint32_t v = 0u;
            if (r < tc.nrows) v = *reinterpret_cast<const uint32_t*>(src + r * mask_ld + pc * 4);
            *reinterpret_cast<uint32_t*>(mtile + r * mstride + pc * 4) = v;
        }
    } else {
        for (int32_t i = threadIdx.x; i < TILE_ROWS * mb; i += blockDim.x) {
            const int32_t r = i / mb, bb = i - r * mb;
            mtile[r * mstride + bb] = r < tc.nrows ? src[r * mask_ld + bb] : (uint8_t)0;
        }
    }
}

// Eight consecutive weights of a lane's row, starting at column c (a multiple of 8).
template <int DT>
__device__ __forceinline__ void read8(const char* __restrict__ wrow, int32_t c, float (&w)[8]) {
    if (DT == WINDQ_BF16) {
        const uint4 raw = *reinterpret_cast<const uint4*>(wrow + c * 2);
        w[0] = bf16_bits_to_f32(raw.x & 0xffffu); w[1] = __uint_as_float(raw.x & 0xffff0000u);
        w[2] = bf16_bits_to_f32(raw.y & 0xffffu); w[3] = __uint_as_float(raw.y & 0xffff0000u);
        w[4] = bf16_bits_to_f32(raw.z & 0xffffu); w[5] = __uint_as_float(raw.z & 0xffff0000u);
        w[6] = bf16_bits_to_f32(raw.w & 0xffffu); w[7] = __uint_as_float(raw.w & 0xffff0000u);
    } else {
        const float4 a = *reinterpret_cast<const float4*>(wrow + c * 4);
        const float4 b = *reinterpret_cast<const float4*>(wrow + c * 4 + 16);
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
        w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    }
}

// Four consecutive weights of a lane's row, starting at column c (a multiple of 4).
template <int DT>
__device__ __forceinline__ void read4(const char* __restrict__ wrow, int32_t c, float (&w)[4]) {
    if (DT == WINDQ_BF16) {
        const uint2 raw = *reinterpret_cast<const uint2*>(wrow + c * 2);
        w[0] = bf16_bits_to_f32(raw.x & 0xffffu); w[1] = __uint_as_float(raw.x & 0xffff0000u);
        w[2] = bf16_bits_to_f32(raw.y & 0xffffu); w[3] = __uint_as_float(raw.y & 0xffff0000u);
    } else {
        const float4 a = *reinterpret_cast<const float4*>(wrow + c * 4);
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    }
}

// Keeps a value in a VGPR and hides its origin from the optimiser, so that it is never
// folded into an SGPR, literal or negated operand (any of which drops the instruction
// to the slow issue rate).
__device__ __forceinline__ float pin_vgpr(float x) {
    asm volatile("" : "+v"(x));
    return x;
}

// a * b + c with the result clamped to [0, 1] by the instruction's output modifier.
__device__ __forceinline__ float fma_clamp01(float a, float b, float c) {
    float r;
    asm("v_fma_f32 %0, %1, %2, %3 clamp" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// a * b with the result clamped to [0, 1] by the instruction's output modifier.
__device__ __forceinline__ float mul_clamp01(float a, float b) {
    float r;
    asm("v_mul_f32 %0, %1, %2 clamp" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Sum of a double over the 64 lanes of a wavefront, fixed butterfly order.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Batched launches number their items (tiles, workgroups, units, strips) one matrix after the
// other; start[i] is the first item of matrix i and start[n] the grid size.  Which matrix holds
// item idx: a scan over at most WINDQ_MAX_BATCH scalars.
__device__ __forceinline__ int batch_index(const int64_t (&start)[WINDQ_MAX_BATCH + 1], int32_t n, int64_t idx) {
    int mi = 0;
    while (mi + 1 < n && idx >= start[mi + 1]) ++mi;
    return mi;
}

// Sum of the n fp64 partials of one unit by a workgroup of NT threads, in a fixed order:
// thread t adds entries t, t + NT, ...; lanes by butterfly, wavefronts in order.  Every
// thread returns the total.
template <int NT>
__device__ __forceinline__ double unit_partial_sum(const double* __restrict__ part, int64_t n, double* red) {
    double t = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += NT) t += part[i];
    t = wave_sum(t);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) tot += red[w];
    return tot;
}

#endif  // __HIPCC__

}  // namespace windq
