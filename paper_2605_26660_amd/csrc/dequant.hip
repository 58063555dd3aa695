// windq_dequant_plan: the way back from the packed artefact.  Unpacks the codes of a plan,
// reconstructs every weight from the stored per-group scale and offset, and recomputes the
// activation-weighted reconstruction error per unit from the artefact alone: the same number
// windq_fit_score_all_bits reported for the plan's bit-width and clip index (Sec. 3.5 scores a
// fit by its reconstruction error; this closes the loop codes -> error), and the first piece of
// a path that serves the quantized weights.
//   uniform:  w_hat = offset + code * scale     ternary: scale * (trit - 1)     binary: +-scale
// Errors use w_hat in fp64 from the stored fp32 numbers, as the fit does; the optional fp32
// output is one fused multiply-add.  Reads 2 bytes per weight plus the codes.
// Two kernels.  Chunk widths of 8 x 2^k columns: a lane owns eight columns of a row, i.e. one
// 16-byte piece of W, one mask byte, `bits` bytes of codes (ternary: the two or three bytes
// its eight trits sit in), and G/8 neighbouring lanes cover a row with contiguous loads
// straight from HBM; a workgroup walks the 64 rows of a tile, each lane keeping the fp64
// weights s_c^2 of its columns.  ~6 fp64 operations per weight: the fp64 ALU and HBM are
// both a few times under their limits.  Other widths: one wavefront per tile, one lane per
// row over a tile staged in LDS (a lane walks its row's byte stream).
#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

struct DequantArgs {
    const void* W;
    const float* s;
    const uint8_t* mask;       // or null
    int64_t mask_ld;
    const uint8_t* action;
    const int64_t* code_off;
    const uint8_t* codes;
    int64_t codes_bytes;
    const float* scale;
    const float* offset;
    Geometry g;
    float* what;               // [rows][what_ld] or null
    int64_t what_ld;
    double* part;              // [n_tiles] or [n_tiles][passes]
    float* err;                // [U] or null
    int64_t per_unit;          // partials per unit
    // matrix-vector product from the artefact (the GEMV kernels), else unused
    const float* x;            // [cols]
    float* y;                  // [rows]
    double* gpart;             // [n_chunks][rows]  a row's partial product over each chunk
};

// A launch covers up to WINDQ_MAX_BATCH matrices (one chunk width, one element type): their
// tiles and units are numbered one matrix after the other.
struct DequantBatch {
    int32_t n;
    int64_t tile_start[WINDQ_MAX_BATCH + 1];
    int64_t unit_start[WINDQ_MAX_BATCH + 1];
    int64_t row_start[WINDQ_MAX_BATCH + 1];
    DequantArgs m[WINDQ_MAX_BATCH];
};

__device__ __forceinline__ int64_t dq_bytes_per_group(int a, int G) {
    switch (a) {
        case 1: return G;
        case 2: return G >> 1;
        case 3: return (G * 3) >> 3;
        case 4: return G >> 2;
        case 5: return (G + 4) / 5;
        case 6: return G >> 3;
        default: return 0;
    }
}

// GEMV: instead of the error and the reconstruction, the product of the reconstruction with x:
// per row and chunk, eight columns at a time in fp32 (fused multiply-adds in column order), those
// runs summed in fp64.
template <int DT, bool GEMV>
__global__ __launch_bounds__(64) void dequant_tile_kernel(const DequantBatch B) {
    extern __shared__ char smem[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const DequantArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
    const int32_t G = A.g.chunk_w;
    constexpr int EB = Elem<DT>::bytes;
    const int32_t row_bytes = G * EB + 16;
    float* scol = reinterpret_cast<float*>(smem + TILE_ROWS * row_bytes);
    const int lane = threadIdx.x;
    load_tile_raw<DT>(A.W, A.g.ld, tc, G, smem);
    for (int32_t c = lane; c < G; c += 64) scol[c] = GEMV ? A.x[tc.col0 + c] : A.s[tc.col0 + c];
    __syncthreads();

    int a = A.action[tc.u];
    if (a >= WINDQ_N_ACTIONS) a = 0;
    const int64_t bpg = dq_bytes_per_group(a, G);
    const int64_t base = A.code_off[tc.u];
    if (base < 0 || (base & 15) != 0 || base + bpg * A.g.R_u > A.codes_bytes) a = 0;   // a malformed entry reads nothing

    double acc = 0.0;
    if (lane < tc.nrows) {
        const char* wrow = smem + lane * row_bytes;
        const int64_t row = tc.row0 + lane;
        const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + lane;
        const float sc = a != 0 ? A.scale[gidx] : 0.0f;
        const float of = a != 0 ? A.offset[gidx] : 0.0f;
        const uint8_t* __restrict__ src = A.codes + base + (tc.lrow0 + lane) * bpg;
        const uint8_t* __restrict__ mrow = A.mask != nullptr ? A.mask + row * A.mask_ld + (tc.col0 >> 3) : nullptr;
        float* __restrict__ orow = !GEMV && A.what != nullptr ? A.what + row * A.what_ld + tc.col0 : nullptr;
        const int bits = a == 1 ? 8 : (a == 2 ? 4 : (a == 3 ? 3 : (a == 4 ? 2 : 1)));
        for (int32_t c = 0; c < G; c += 8) {
            float w[8];
            read8<DT>(wrow, c, w);
            const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
            uint32_t stored[8];
            if (a == 5) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int32_t i = c + j;
                    const uint32_t byte = src[i / 5];
                    const int pos = i % 5;
                    const uint32_t div = pos == 0 ? 1u : (pos == 1 ? 3u : (pos == 2 ? 9u : (pos == 3 ? 27u : 81u)));
                    stored[j] = (byte / div) % 3u;
                }
            } else if (a != 0) {
                uint64_t v = 0;
                const uint8_t* p = src + (c >> 3) * bits;          // eight codes = `bits` bytes
                for (int b = 0; b < bits; ++b) v |= (uint64_t)p[b] << (8 * b);
#pragma unroll
                for (int j = 0; j < 8; ++j) stored[j] = (uint32_t)(v >> (j * bits)) & ((1u << bits) - 1u);
            }
            float run = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool prot = ((m >> j) & 1u) != 0u;
                float wh = w[j];                                      // a skip unit keeps its weights
                if (a != 0) {
                    double whd;
                    if (a <= 4) {
                        wh = fmaf((float)stored[j], sc, of);
                        whd = (double)of + (double)stored[j] * (double)sc;
                    } else if (a == 5) {
                        wh = sc * ((float)stored[j] - 1.0f);
                        whd = (double)wh;
                    } else {
                        wh = stored[j] != 0u ? sc : -sc;
                        whd = (double)wh;
                    }
                    if (prot) {
                        wh = 0.0f;                                    // lives in the INT8 side stream
                    } else if (!GEMV) {
                        const double d = (double)w[j] - whd;
                        const double ac = (double)scol[c + j] * (double)scol[c + j];
                        acc = fma(ac * d, d, acc);
                    }
                }
                if (GEMV) run = fmaf(wh, scol[c + j], run);
                else if (orow != nullptr) orow[c + j] = wh;
            }
            if (GEMV) acc += (double)run;
        }
        if (GEMV) A.gpart[(tc.col0 / G) * A.g.rows + row] = acc;
    }
    if (GEMV) return;
    acc = wave_sum(acc);
    if (lane == 0) A.part[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] = acc;      // one partial per tile
}

// Eight consecutive weights of a row, straight from global memory.
template <int DT>
__device__ __forceinline__ void load8_global(const void* __restrict__ p, float (&w)[8]) {
    if (DT == WINDQ_BF16) {
        const uint4 raw = *reinterpret_cast<const uint4*>(p);
        w[0] = bf16_bits_to_f32(raw.x & 0xffffu); w[1] = __uint_as_float(raw.x & 0xffff0000u);
        w[2] = bf16_bits_to_f32(raw.y & 0xffffu); w[3] = __uint_as_float(raw.y & 0xffff0000u);
        w[4] = bf16_bits_to_f32(raw.z & 0xffffu); w[5] = __uint_as_float(raw.z & 0xffff0000u);
        w[6] = bf16_bits_to_f32(raw.w & 0xffffu); w[7] = __uint_as_float(raw.w & 0xffff0000u);
    } else {
        const float4 a = reinterpret_cast<const float4*>(p)[0];
        const float4 b = reinterpret_cast<const float4*>(p)[1];
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
        w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    }
}

// Lanes-per-row kernel: chunk_w = 8 << lpr_shift columns.  A workgroup takes one pass of a
// 64-row tile, the 256 >> lpr_shift rows its threads cover at once: no loop over rows, so all
// of a workgroup's loads are in flight together.
constexpr int DQ_THREADS = 256;
template <int DT, bool GEMV>
__global__ __launch_bounds__(DQ_THREADS) void dequant_split_kernel(const DequantBatch B, const int lpr_shift) {
    __shared__ double red[DQ_THREADS / 64];
    const int32_t passes = dequant_passes(8 << lpr_shift);
    // (the product: a workgroup takes all passes of its tile, one after the other, and keeps its x)
    const int64_t tile_b = GEMV ? (int64_t)blockIdx.x : blockIdx.x / passes;                 // tile of the launch
    const int32_t pass0 = GEMV ? 0 : (int32_t)(blockIdx.x - tile_b * passes);
    const int mi = batch_index(B.tile_start, B.n, tile_b);
    const DequantArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, tile_b - B.tile_start[mi]);
    const int32_t G = A.g.chunk_w;
    constexpr int EB = Elem<DT>::bytes;
    const int sub = threadIdx.x & ((1 << lpr_shift) - 1);      // which 8 columns of the row
    const int rsub = threadIdx.x >> lpr_shift;                 // which row of a pass
    const int rows_per_pass = DQ_THREADS >> lpr_shift;
    const int32_t c = sub * 8;

    int a = A.action[tc.u];
    if (a >= WINDQ_N_ACTIONS) a = 0;
    const int64_t bpg = dq_bytes_per_group(a, G);
    const int64_t base = A.code_off[tc.u];
    if (base < 0 || (base & 15) != 0 || base + bpg * A.g.R_u > A.codes_bytes) a = 0;   // a malformed entry reads nothing
    const int bits = a == 1 ? 8 : (a == 2 ? 4 : (a == 3 ? 3 : (a == 4 ? 2 : 1)));

    double ac[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const double sv = GEMV ? 0.0 : (double)A.s[tc.col0 + c + j];
        ac[j] = sv * sv;
    }
    // ternary: a byte's five trits as five 2-bit fields, from a table the workgroup fills once
    __shared__ uint16_t trits_of[256];
    if (a == 5) {
        uint32_t b = threadIdx.x, t = 0;
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            t |= (b % 3u) << (2 * i);
            b /= 3u;
        }
        trits_of[threadIdx.x] = (uint16_t)t;
        __syncthreads();
    }

    float xv[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    if (GEMV) {
#pragma unroll
        for (int j = 0; j < 8; ++j) xv[j] = A.x[tc.col0 + c + j];
    }
    double acc = 0.0;
    for (int32_t pass = pass0; pass < (GEMV ? passes : pass0 + 1); ++pass) {
        float dot = 0.0f;           // GEMV: this thread's eight columns of the row times x
        const int32_t r = pass * rows_per_pass + rsub;
        if (r < tc.nrows && r < TILE_ROWS) {
            const int64_t row = tc.row0 + r;
            const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + r;
            float w[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
            if (!GEMV || a == 0)        // the product reads W only for skip units
                load8_global<DT>(static_cast<const char*>(A.W) + (row * A.g.ld + tc.col0 + c) * EB, w);
            const uint32_t m = A.mask != nullptr ? A.mask[row * A.mask_ld + (tc.col0 >> 3) + sub] : 0u;
            float* __restrict__ orow = !GEMV && A.what != nullptr ? A.what + row * A.what_ld + tc.col0 + c : nullptr;
            float wh[8];
            if (a == 0) {
#pragma unroll
                for (int j = 0; j < 8; ++j) wh[j] = w[j];                     // a skip unit keeps its weights
            } else {
                const float sc = A.scale[gidx];
                const float of = A.offset[gidx];
                const uint8_t* __restrict__ src = A.codes + base + (tc.lrow0 + r) * bpg;
                double whd[8];
                if (a == 5) {
                    // eight trits, five to a byte: they sit in two or three neighbouring bytes
                    const int32_t b0 = c / 5;
                    const int32_t last = (int32_t)bpg - 1;
                    const uint32_t y0 = src[b0];
                    const uint32_t y1 = src[b0 + 1 <= last ? b0 + 1 : last];
                    const uint32_t y2 = src[b0 + 2 <= last ? b0 + 2 : last];
                    const uint32_t v = ((uint32_t)trits_of[y0] | ((uint32_t)trits_of[y1] << 10) | ((uint32_t)trits_of[y2] << 20)) >>
                                       (2 * (c - 5 * b0));
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        wh[j] = sc * ((float)((v >> (2 * j)) & 3u) - 1.0f);
                        whd[j] = (double)wh[j];
                    }
                } else {
                    // eight codes = `bits` bytes, aligned to their own size (units start on 16 bytes)
                    const uint8_t* p = src + sub * bits;
                    uint64_t v;
                    if (bits == 8) {
                        const uint2 t = *reinterpret_cast<const uint2*>(p);
                        v = (uint64_t)t.x | ((uint64_t)t.y << 32);
                    } else if (bits == 4) {
                        v = *reinterpret_cast<const uint32_t*>(p);
                    } else if (bits == 3) {
                        const uint32_t t0 = p[0], t1 = p[1], t2 = p[2];
                        v = t0 | (t1 << 8) | (t2 << 16);
                    } else if (bits == 2) {
                        v = *reinterpret_cast<const uint16_t*>(p);
                    } else {
                        v = p[0];
                    }
                    if (a == 6) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            wh[j] = ((v >> j) & 1u) != 0u ? sc : -sc;
                            whd[j] = (double)wh[j];
                        }
                    } else {
                        const double scd = (double)sc, ofd = (double)of;
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const uint32_t code = (uint32_t)(v >> (j * bits)) & ((1u << bits) - 1u);
                            wh[j] = fmaf((float)code, sc, of);
                            whd[j] = ofd + (double)code * scd;
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool prot = ((m >> j) & 1u) != 0u;              // lives in the INT8 side stream
                    if (!GEMV) {
                        const double d = (double)w[j] - whd[j];
                        acc = fma(prot ? 0.0 : ac[j] * d, d, acc);
                    }
                    wh[j] = prot ? 0.0f : wh[j];
                }
            }
            if (GEMV) {
#pragma unroll
                for (int j = 0; j < 8; ++j) dot = fmaf(wh[j], xv[j], dot);
            } else if (orow != nullptr) {
                reinterpret_cast<float4*>(orow)[0] = make_float4(wh[0], wh[1], wh[2], wh[3]);
                reinterpret_cast<float4*>(orow)[1] = make_float4(wh[4], wh[5], wh[6], wh[7]);
            }
        }
        if (GEMV) {
            // the row's 8-column runs, held by neighbouring lanes, summed in fp64
            double d = (double)dot;
            for (int mk = 1; mk < (1 << lpr_shift); mk <<= 1) d += __shfl_xor(d, mk, 64);
            if (sub == 0 && r < tc.nrows && r < TILE_ROWS) A.gpart[(tc.col0 / G) * A.g.rows + tc.row0 + r] = d;
        }
    }
    if (GEMV) return;
    const int32_t pass = pass0;
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int i = 0; i < DQ_THREADS / 64; ++i) t += red[i];
        A.part[((size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t) * (size_t)passes + (size_t)pass] = t;
    }
}

// err[u] = the sum of unit u's per_unit partials; one workgroup per unit.
__global__ __launch_bounds__(256) void dequant_finalize_kernel(const DequantBatch B) {
    __shared__ double red[4];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const DequantArgs& A = B.m[mi];
    if (A.err == nullptr) return;
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    const double t = unit_partial_sum<256>(A.part + (size_t)u * (size_t)A.per_unit, A.per_unit, red);
    if (threadIdx.x == 0) A.err[u] = (float)t;
}

// y[row] = the row's chunk partials in chunk order, fp64, rounded once; one thread per row.
__global__ __launch_bounds__(256) void dequant_gemv_finalize_kernel(const DequantBatch B) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= B.row_start[B.n]) return;
    const int mi = batch_index(B.row_start, B.n, i);
    const DequantArgs& A = B.m[mi];
    const int64_t row = i - B.row_start[mi];
    double t = 0.0;
    for (int64_t j0 = 0; j0 < A.g.n_chunks; j0 += 8) {       // eight loads in flight, added in chunk order
        double v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = j0 + k < A.g.n_chunks ? A.gpart[(j0 + k) * A.g.rows + row] : 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += v[k];
    }
    A.y[row] = (float)t;
}

// Numbers the tiles and units of the first B->n matrices.
static int64_t dequant_number(DequantBatch* B) {
    int64_t tiles = 0, units = 0, rows = 0;
    for (int32_t i = 0; i < B->n; ++i) {
        B->tile_start[i] = tiles;
        B->unit_start[i] = units;
        B->row_start[i] = rows;
        tiles += B->m[i].g.n_tiles;
        units += B->m[i].g.U;
        rows += B->m[i].g.rows;
    }
    for (int32_t i = B->n; i <= WINDQ_MAX_BATCH; ++i) {
        B->tile_start[i] = tiles;
        B->unit_start[i] = units;
        B->row_start[i] = rows;
    }
    for (int32_t i = B->n; i < WINDQ_MAX_BATCH; ++i) B->m[i] = B->m[0];
    return tiles;
}

}  // namespace windq

using namespace windq;

// One matrix of a launch as the entry points see it (the check call, or the product when x is set).
struct DequantItem {
    const windq_mat* W;
    const float* s;
    const uint8_t* mask;
    const uint8_t* action;
    const int64_t* code_off;
    const uint8_t* codes;
    size_t codes_bytes;
    const float* scale;
    const float* offset;
    float* err;
    float* w_hat;
    const float* x;
    float* y;
    void* ws;
    size_t ws_bytes;
};

// Matrices whose layout allows it go through the lanes-per-row kernel, the others through the
// tile kernel, exactly as each would alone: at most two sub-batches per call.
template <bool GEMV>
static int dequant_launch(const DequantItem* items, int32_t n, int32_t chunk_w, int64_t unit_rows, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    // lanes-per-row kernel: 8 x 2^k columns, 16-byte pieces of W and of w_hat aligned
    int lpr_shift = -1;
    for (int k = 0; k <= 6; ++k)
        if (chunk_w == (8 << k)) lpr_shift = k;
    const int32_t passes = dequant_passes(chunk_w);
    DequantBatch S, T;          // lanes-per-row, tile
    S.n = T.n = 0;
    bool any_err_s = false, any_err_t = false;
    for (int32_t i = 0; i < n; ++i) {
        const DequantItem& it = items[i];
        DequantArgs A;
        if (it.W == nullptr) return WINDQ_EINVAL;
        const int st = make_geometry(it.W, chunk_w, unit_rows, &A.g);
        if (st != WINDQ_OK) return st;
        if (it.action == nullptr || it.code_off == nullptr || it.scale == nullptr || it.offset == nullptr) return WINDQ_EINVAL;
        if (it.codes == nullptr && it.codes_bytes != 0) return WINDQ_EINVAL;
        if (GEMV) {
            if (it.x == nullptr || it.y == nullptr) return WINDQ_EINVAL;
        } else {
            if (it.s == nullptr || (it.err == nullptr && it.w_hat == nullptr)) return WINDQ_EINVAL;
            if (it.w_hat != nullptr && !aligned(it.w_hat, 4)) return WINDQ_EINVAL;
        }
        if (!aligned(it.code_off, 8)) return WINDQ_EINVAL;
        if (it.W->dtype != items[0].W->dtype) return WINDQ_EINVAL;      // one kernel per launch
        const size_t need = GEMV ? dequant_gemv_ws_bytes(A.g) : dequant_ws_bytes(A.g);
        if (it.ws == nullptr || it.ws_bytes < need || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        A.W = it.W->data;
        A.s = it.s;
        A.mask = it.mask;
        A.mask_ld = it.W->cols / 8;
        A.action = it.action;
        A.code_off = it.code_off;
        A.codes = it.codes;
        A.codes_bytes = (int64_t)it.codes_bytes;
        A.scale = it.scale;
        A.offset = it.offset;
        A.what = GEMV ? nullptr : it.w_hat;
        A.what_ld = it.W->cols;
        A.part = static_cast<double*>(it.ws);
        A.err = GEMV ? nullptr : it.err;
        A.x = it.x;
        A.y = it.y;
        A.gpart = static_cast<double*>(it.ws);
        const size_t eb = it.W->dtype == WINDQ_BF16 ? 2 : 4;
        const bool split = lpr_shift >= 0 && aligned(it.W->data, 16) && ((size_t)it.W->ld * eb) % 16 == 0 &&
                           (A.what == nullptr || aligned(A.what, 16)) && aligned(it.codes, 8);
        A.per_unit = split ? A.g.tiles_per_unit * passes : A.g.tiles_per_unit;
        if (split) {
            S.m[S.n++] = A;
            any_err_s = any_err_s || A.err != nullptr;
        } else {
            T.m[T.n++] = A;
            any_err_t = any_err_t || A.err != nullptr;
        }
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t dtype = items[0].W->dtype;
    if (S.n > 0) {
        const int64_t tiles = dequant_number(&S);
        if (tiles * passes > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
        const dim3 grid((unsigned)(GEMV ? tiles : tiles * passes));
        if (dtype == WINDQ_BF16) hipLaunchKernelGGL((dequant_split_kernel<WINDQ_BF16, GEMV>), grid, dim3(DQ_THREADS), 0, hs, S, lpr_shift);
        else hipLaunchKernelGGL((dequant_split_kernel<WINDQ_F32, GEMV>), grid, dim3(DQ_THREADS), 0, hs, S, lpr_shift);
        if (GEMV) hipLaunchKernelGGL(dequant_gemv_finalize_kernel, dim3((unsigned)((S.row_start[S.n] + 255) / 256)), dim3(256), 0, hs, S);
        else if (any_err_s) hipLaunchKernelGGL(dequant_finalize_kernel, dim3((unsigned)S.unit_start[S.n]), dim3(256), 0, hs, S);
    }
    if (T.n > 0) {
        const int64_t tiles = dequant_number(&T);
        if (tiles > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
        const size_t lds = raw_tile_lds_bytes(dtype, chunk_w) + (size_t)chunk_w * sizeof(float);
        const dim3 grid((unsigned)tiles);
        if (dtype == WINDQ_BF16) {
            const int st = ensure_lds(reinterpret_cast<const void*>(&dequant_tile_kernel<WINDQ_BF16, GEMV>), lds);
            if (st != WINDQ_OK) return st;
            hipLaunchKernelGGL((dequant_tile_kernel<WINDQ_BF16, GEMV>), grid, dim3(64), lds, hs, T);
        } else {
            const int st = ensure_lds(reinterpret_cast<const void*>(&dequant_tile_kernel<WINDQ_F32, GEMV>), lds);
            if (st != WINDQ_OK) return st;
            hipLaunchKernelGGL((dequant_tile_kernel<WINDQ_F32, GEMV>), grid, dim3(64), lds, hs, T);
        }
        if (GEMV) hipLaunchKernelGGL(dequant_gemv_finalize_kernel, dim3((unsigned)((T.row_start[T.n] + 255) / 256)), dim3(256), 0, hs, T);
        else if (any_err_t) hipLaunchKernelGGL(dequant_finalize_kernel, dim3((unsigned)T.unit_start[T.n]), dim3(256), 0, hs, T);
    }
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

extern "C" int windq_dequant_plan(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                  const uint8_t* mask, const uint8_t* action, const int64_t* code_off,
                                  const uint8_t* codes, size_t codes_bytes, const float* scale, const float* offset,
                                  float* err, float* w_hat, void* ws, size_t ws_bytes, void* stream) {
    const DequantItem it = {W, s, mask, action, code_off, codes, codes_bytes, scale, offset, err, w_hat, nullptr, nullptr, ws, ws_bytes};
    return dequant_launch<false>(&it, 1, chunk_w, unit_rows, stream);
}

extern "C" int windq_dequant_plan_batch(const windq_dequant_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                        void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    DequantItem its[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i)
        its[i] = {items[i].W, items[i].s, items[i].mask, items[i].action, items[i].code_off, items[i].codes, items[i].codes_bytes,
                  items[i].scale, items[i].offset, items[i].err, items[i].w_hat, nullptr, nullptr, items[i].ws, items[i].ws_bytes};
    return dequant_launch<false>(its, n, chunk_w, unit_rows, stream);
}

extern "C" int windq_dequant_gemv(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, const uint8_t* mask,
                                  const uint8_t* action, const int64_t* code_off, const uint8_t* codes, size_t codes_bytes,
                                  const float* scale, const float* offset, const float* x, float* y, void* ws,
                                  size_t ws_bytes, void* stream) {
    const DequantItem it = {W, nullptr, mask, action, code_off, codes, codes_bytes, scale, offset, nullptr, nullptr, x, y, ws, ws_bytes};
    return dequant_launch<true>(&it, 1, chunk_w, unit_rows, stream);
}

extern "C" int windq_dequant_gemv_batch(const windq_gemv_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                        void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    DequantItem its[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i)
        its[i] = {items[i].W, nullptr, items[i].mask, items[i].action, items[i].code_off, items[i].codes, items[i].codes_bytes,
                  items[i].scale, items[i].offset, nullptr, nullptr, items[i].x, items[i].y, items[i].ws, items[i].ws_bytes};
    return dequant_launch<true>(its, n, chunk_w, unit_rows, stream);
}
