// HiF4 encoder (Algorithm 1, Section II-B of the HiF4 paper) and decoder (Eq. 2,
// Section II-A) for gfx950.  Both are HBM-bound streaming kernels: 128 B of BF16
// against 36 B of packed unit.
//
// Work split: a unit of 64 elements is shared by LPU adjacent lanes; every lane owns
// 8/LPU "chunks" of 8 consecutive elements (one 128-bit load each, one level-2
// micro-exponent domain, two level-3 domains).  The peak magnitude of the unit and
// the metadata bits are exchanged across the LPU lanes with DPP moves; nothing goes
// through LDS.
#include "hif4_encode.h"
#include "hif4_expand.h"

namespace hif4 {

// ------------------------------------------------------------------ encoder

// Input element types of the encoder.  FP16 and FP32 inputs are first rounded to BF16 by the
// rounding mode of the conversion (Section II-B: other high-precision formats follow the same
// procedure; Algorithm 1 itself is written on BF16), then take the same path.
enum { IN_BF16 = 0, IN_F16 = 1, IN_F32 = 2 };

// One exact fp32 value -> BF16 pattern under MODE; NaNs stay NaNs, overflow gives infinity.
template <int MODE>
__device__ __forceinline__ uint32_t input_pair_to_bf16(float lo, float hi)
{
    if (MODE == HIF4_ROUND_RNE) return round_bf16_pair<MODE>(lo, hi); // v_cvt_pk_bf16_f32 keeps NaN and Inf
    uint32_t r[2];
    const uint32_t u[2] = { f2u(lo), f2u(hi) };
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t a = u[i] & 0x7FFFFFFFu;
        const uint32_t m = a > 0x7F800000u ? 0x7FC0u : (a + 0x8000u) >> 16; // magnitude, half away from zero
        r[i] = m | ((u[i] >> 16) & 0x8000u);
    }
    return r[0] | (r[1] << 16);
}

// 8 consecutive input elements starting at element index e of x -> 8 BF16 in a uint4.
template <int IN, int MODE, bool NT>
__device__ __forceinline__ uint4 load_chunk(const void *x, int64_t e)
{
    if (IN == IN_BF16) return load16<NT>(static_cast<const uint16_t *>(x) + e);
    if (IN == IN_F16) {
        const uint4 h = load16<NT>(static_cast<const uint16_t *>(x) + e);
        const uint32_t hw[4] = { h.x, h.y, h.z, h.w };
        uint32_t r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            const h2 v = __builtin_bit_cast(h2, hw[t]);
            r[t] = input_pair_to_bf16<MODE>((float)v.x, (float)v.y); // FP16 -> fp32 is exact
        }
        return make_uint4(r[0], r[1], r[2], r[3]);
    }
    const float *f = static_cast<const float *>(x) + e;
    const uint4 a = load16<NT>(f), b = load16<NT>(f + 4);
    return make_uint4(input_pair_to_bf16<MODE>(u2f(a.x), u2f(a.y)), input_pair_to_bf16<MODE>(u2f(a.z), u2f(a.w)),
                      input_pair_to_bf16<MODE>(u2f(b.x), u2f(b.y)), input_pair_to_bf16<MODE>(u2f(b.z), u2f(b.w)));
}

// Thread block b encodes units [b * UPB, (b+1) * UPB), UPB = UPT * 256 / LPU; a thread's
// t-th unit is UPB*b + t*(256/LPU) + threadIdx/LPU, so that every load and store
// instruction of a wave touches one contiguous range.
template <int LPU, int MODE, bool CONTIG, int UPT, bool NT, int IN = IN_BF16>
__global__ __launch_bounds__(256) void encode_kernel(const void *__restrict__ x, int64_t units, int64_t upr,
                                                     int64_t ldx, uint32_t *__restrict__ codes,
                                                     uint32_t *__restrict__ meta)
{
    constexpr int NCH = 8 / LPU;
    constexpr int UPS = 256 / LPU; // units per block per slice
    const int l = (int)(threadIdx.x % LPU);
    const int64_t first = (int64_t)blockIdx.x * (UPS * UPT) + threadIdx.x / LPU;

    uint4 w[UPT][NCH];
    int64_t unit[UPT];
    bool live[UPT];
#pragma unroll
    for (int t = 0; t < UPT; ++t) {
        const int64_t u = first + (int64_t)t * UPS;
        live[t] = u < units;
        unit[t] = live[t] ? u : units - 1; // dead lanes redo the last unit and store nothing
        int64_t e0; // index of the unit's first element in x
        if (CONTIG) {
            e0 = unit[t] * 64;
        } else {
            const int64_t row = unit[t] / upr;
            e0 = row * ldx + (unit[t] - row * upr) * 64;
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) w[t][c] = load_chunk<IN, MODE, NT>(x, e0 + 8 * (c * LPU + l));
    }
#pragma unroll
    for (int t = 0; t < UPT; ++t) {
        uint32_t out[NCH];
        const uint32_t m = encode_share<LPU, MODE>(w[t], l, out);
        if (live[t]) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) store4<NT>(codes + unit[t] * 8 + c * LPU + l, out[c]);
            if (l == 0) store4<NT>(meta + unit[t], m);
        }
    }
}

// Quantise-dequantise in one pass for the GEMM that converts its activations itself: the same
// loads and the same Algorithm 1 as encode_kernel, but what is stored is the exact BF16 value of
// every element of the resulting unit (Eq. 2), 8 per 16-byte cell in the cell order of the tile
// GEMM, dense rows.  The packed unit never goes to memory.  NATURAL: every group of 8 in element order
// instead (plain decoded rows, what hif4_dequantize would write).
template <int MODE, bool CONTIG, bool NATURAL = false>
__global__ __launch_bounds__(256) void encode_to_cells_kernel(const void *__restrict__ x, int64_t units, int64_t upr,
                                                              int64_t ldx, uint4 *__restrict__ cells)
{
    constexpr int LPU = 4, NCH = 2;
    const int l = (int)(threadIdx.x % LPU);
    const int64_t u = (int64_t)blockIdx.x * (256 / LPU) + threadIdx.x / LPU;
    const bool live = u < units;
    const int64_t unit = live ? u : units - 1; // dead lanes redo the last unit and store nothing
    int64_t e0;
    if (CONTIG) {
        e0 = unit * 64;
    } else {
        const int64_t row = unit / upr;
        e0 = row * ldx + (unit - row * upr) * 64;
    }
    uint4 w[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) w[c] = load_chunk<IN_BF16, MODE, false>(x, e0 + 8 * (c * LPU + l));
    uint32_t out[NCH];
    const uint32_t m = encode_share<LPU, MODE>(w, l, out);
    const uint32_t sbase = unit_scale_bits(m);
    if (live) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            cells[unit * 8 + c * LPU + l] = NATURAL ? decode_chunk(out[c], m, c * LPU + l) : expand_chunk(out[c], m, sbase, c * LPU + l);
    }
}

// The same, stored as "cell planes" (cell (row, group g of 8 along K) at index g * rows + row: the
// layout the plane-fed GEMM kernels load straight into LDS).  A block takes one unit of 64
// consecutive rows, four lanes per unit, so that the 16 lanes of a wave that hold the same group
// write 256 consecutive bytes of its plane.
template <int MODE>
__global__ __launch_bounds__(256) void encode_to_planes_kernel(const void *__restrict__ x, int64_t rows, int64_t ldx,
                                                               uint4 *__restrict__ planes)
{
    constexpr int LPU = 4, NCH = 2;
    const int l = (int)(threadIdx.x % LPU);
    // one grid axis (row blocks fastest): K is not bounded by the 65535 blocks of a second axis
    const int64_t row_blocks = (rows + 63) / 64;
    const int64_t r = (int64_t)(blockIdx.x % row_blocks) * 64 + threadIdx.x / LPU, u = blockIdx.x / row_blocks;
    const bool live = r < rows;
    const int64_t row = live ? r : rows - 1; // dead lanes redo the last row and store nothing
    const int64_t e0 = row * ldx + u * 64;
    uint4 w[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) w[c] = load_chunk<IN_BF16, MODE, false>(x, e0 + 8 * (c * LPU + l));
    uint32_t out[NCH];
    const uint32_t m = encode_share<LPU, MODE>(w, l, out);
    const uint32_t sbase = unit_scale_bits(m);
    if (live) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) planes[(u * 8 + c * LPU + l) * rows + row] = expand_chunk(out[c], m, sbase, c * LPU + l);
    }
}

int launch_encode_to_planes(const void *x, int64_t rows, int64_t K, int64_t ldx, void *planes, int mode, hipStream_t stream)
{
    const int64_t upr = K / 64;
    if (rows == 0 || upr == 0) return HIF4_OK;
    const int64_t blocks = (rows + 63) / 64 * upr;
    if (blocks > 0x7FFFFFFF) return HIF4_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(256);
    uint4 *y = static_cast<uint4 *>(planes);
    if (mode == HIF4_ROUND_RNE) hipLaunchKernelGGL(encode_to_planes_kernel<HIF4_ROUND_RNE>, grid, block, 0, stream, x, rows, ldx, y);
    else hipLaunchKernelGGL(encode_to_planes_kernel<HIF4_ROUND_RHA>, grid, block, 0, stream, x, rows, ldx, y);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// Quantise and decode in one pass into dense rows of BF16 in natural element order (row stride K).
int launch_encode_to_rows(const void *x, int64_t rows, int64_t K, int64_t ldx, void *y, int mode, hipStream_t stream)
{
    const int64_t upr = K / 64, units = rows * upr;
    if (units == 0) return HIF4_OK;
    const dim3 grid((unsigned)((units + 63) / 64)), block(256);
    uint4 *out = static_cast<uint4 *>(y);
    if (mode == HIF4_ROUND_RNE) hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RNE, false, true>), grid, block, 0, stream, x, units, upr, ldx, out);
    else hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RHA, false, true>), grid, block, 0, stream, x, units, upr, ldx, out);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_encode_to_cells(const void *x, int64_t rows, int64_t K, int64_t ldx, void *cells, int mode, hipStream_t stream)
{
    const int64_t upr = K / 64, units = rows * upr;
    if (units == 0) return HIF4_OK;
    const dim3 grid((unsigned)((units + 63) / 64)), block(256);
    uint4 *y = static_cast<uint4 *>(cells);
    const bool contig = ldx == K;
    if (mode == HIF4_ROUND_RNE) {
        if (contig) hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RNE, true>), grid, block, 0, stream, x, units, upr, ldx, y);
        else hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RNE, false>), grid, block, 0, stream, x, units, upr, ldx, y);
    } else {
        if (contig) hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RHA, true>), grid, block, 0, stream, x, units, upr, ldx, y);
        else hipLaunchKernelGGL((encode_to_cells_kernel<HIF4_ROUND_RHA, false>), grid, block, 0, stream, x, units, upr, ldx, y);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// ------------------------------------------------------------------ decoder

// One lane decodes CPT chunks of 8 elements; block b owns chunks [b*256*CPT, (b+1)*256*CPT).
// CELL: write each group of 8 in the GEMM's cell order (an internal staging format) instead
// of element order.
template <bool CONTIG, int CPT, bool NT, bool CELL = false>
__global__ __launch_bounds__(256) void decode_kernel(const uint32_t *__restrict__ codes,
                                                     const uint32_t *__restrict__ meta, int64_t chunks, int64_t upr,
                                                     int64_t ldy, uint16_t *__restrict__ y)
{
    const int64_t first = (int64_t)blockIdx.x * (256 * CPT) + threadIdx.x;
    uint32_t c[CPT], m[CPT];
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
        const int64_t id = first + t * 256;
        const int64_t idc = id < chunks ? id : chunks - 1;
        c[t] = NT ? __builtin_nontemporal_load(codes + idc) : codes[idc];
        m[t] = meta[idc >> 3];
    }
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
        const int64_t id = first + t * 256;
        if (id >= chunks) continue;
        const int64_t unit = id >> 3;
        const int j = (int)(id & 7);
        uint16_t *dst;
        if (CONTIG) {
            dst = y + id * 8;
        } else {
            const int64_t row = unit / upr;
            dst = y + row * ldy + (unit - row * upr) * 64 + j * 8;
        }
        if (CELL) store16<NT>(dst, expand_chunk(c[t], m[t], unit_scale_bits(m[t]), j));
        else store16<NT>(dst, decode_chunk(c[t], m[t], j));
    }
}

// ------------------------------------------------------------------ launchers

// Launch shapes measured on MI355X at 512 MiB of BF16: 4 lanes per unit and one unit
// slice per thread for the encoder (the kernel is VALU-limited, fewer lanes per unit
// amortise the per-unit scalar work); 4 chunks per thread and streaming stores for the
// decoder (write-dominated).
#ifndef HIF4_ENC_LPU
#define HIF4_ENC_LPU 4
#endif
#ifndef HIF4_ENC_UPT
#define HIF4_ENC_UPT 1
#endif
#ifndef HIF4_ENC_NT
#define HIF4_ENC_NT false
#endif
#ifndef HIF4_DEC_CPT
#define HIF4_DEC_CPT 4
#endif
#ifndef HIF4_DEC_NT
#define HIF4_DEC_NT true
#endif

template <int IN>
static int launch_encode_in(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                            hipStream_t stream)
{
    const int64_t upr = K / 64, units = rows * upr;
    if (units == 0) return HIF4_OK;
    constexpr int LPU = HIF4_ENC_LPU, UPT = HIF4_ENC_UPT;
    constexpr bool NT = HIF4_ENC_NT;
    constexpr int64_t UPB = (256 / LPU) * UPT; // units per block
    const dim3 grid((unsigned)((units + UPB - 1) / UPB)), block(256);
    uint32_t *cd = reinterpret_cast<uint32_t *>(codes);
    const bool contig = ldx == K;
    if (mode == HIF4_ROUND_RNE) {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, true, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, false, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
    } else {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, true, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, false, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_encode(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                  hipStream_t stream)
{
    return launch_encode_in<IN_BF16>(x, rows, K, ldx, codes, meta, mode, stream);
}

// in_dtype: HIF4_IN_BF16 / HIF4_IN_F16 / HIF4_IN_F32 of the C interface (same numbering as above).
int launch_encode_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                       int mode, hipStream_t stream)
{
    if (in_dtype == IN_F16) return launch_encode_in<IN_F16>(x, rows, K, ldx, codes, meta, mode, stream);
    if (in_dtype == IN_F32) return launch_encode_in<IN_F32>(x, rows, K, ldx, codes, meta, mode, stream);
    return launch_encode_in<IN_BF16>(x, rows, K, ldx, codes, meta, mode, stream);
}

int launch_decode(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, int64_t ldy,
                  hipStream_t stream)
{
    const int64_t upr = K / 64, chunks = rows * upr * 8;
    if (chunks == 0) return HIF4_OK;
    constexpr int CPT = HIF4_DEC_CPT;
    constexpr bool NT = HIF4_DEC_NT;
    const dim3 grid((unsigned)((chunks + 256 * CPT - 1) / (256 * CPT))), block(256);
    const uint32_t *cd = reinterpret_cast<const uint32_t *>(codes);
    uint16_t *ys = static_cast<uint16_t *>(y);
    if (ldy == K) hipLaunchKernelGGL((decode_kernel<true, CPT, NT>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    else hipLaunchKernelGGL((decode_kernel<false, CPT, NT>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// HiF4 -> BF16 copy in cell order, dense rows (row stride K): the activation operand of the
// tile GEMM.  Regular stores: the GEMM reads the copy right away.
int launch_decode_cells(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, hipStream_t stream)
{
    const int64_t upr = K / 64, chunks = rows * upr * 8;
    if (chunks == 0) return HIF4_OK;
    constexpr int CPT = HIF4_DEC_CPT;
    const dim3 grid((unsigned)((chunks + 256 * CPT - 1) / (256 * CPT))), block(256);
    hipLaunchKernelGGL((decode_kernel<true, CPT, false, true>), grid, block, 0, stream,
                       reinterpret_cast<const uint32_t *>(codes), meta, chunks, upr, K, static_cast<uint16_t *>(y));
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

} // namespace hif4
