// MXFP4 (packed E2M1 + UE8M0 per 1x32) -> FP8 (E4M3 + FP32 1x128 scales), gfx950.
//
// Paper sec. 3.3, Algorithm 1: the tile scale is max(SF_0..SF_3) - 6 placed into the FP32
// exponent field, and each element's exponent is re-biased (E_fp4 - 1 + 7) and reduced by
// the alignment shift of its block; the mantissa bit moves to the E4M3 mantissa MSB.
// No floating-point arithmetic is involved: per block the map "3-bit magnitude -> E4M3
// byte" is an 8-entry byte table that depends only on d = max(SF) - SF_block, and
// v_perm_b32 looks up four entries per instruction.
//   d <= 11 : every entry is a normal E4M3 number: table(d) = table(0) - 8*d per entry,
//             which is Algorithm 1's exponent subtraction done on four bytes at once.
//   d >= 12 : entries fall into the E4M3 subnormals and round to nearest-even (gradual
//             underflow; exact up to d = 14), all zero from d = 19.  Taken from a small
//             constant table built at compile time.
// The E2M1 codes 0 (zero) and 1 (the subnormal 0.5 = 1.0 * 2^-1) have their own entries.
//
// Work split: one lane owns half a 1x32 block (8-byte load, one 16-byte store), so a wave's
// loads and stores are contiguous; the 8 lanes of a 128-tile agree on max(SF) with two DPP
// exchanges.
// HBM-bound: 0.53125 B read + 1.03125 B written per element.
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

// Cache policy and launch shape, measured at [65536,7168] over rotated buffer sets (every byte from and to HBM).
// Non-temporal loads; the E4M3 bytes, two thirds of the traffic and written in address order by the whole grid,
// leave with streaming stores (store_streaming): 111 us, against 115 us with the non-temporal hint alone and
// 114 us with plain loads.  The 4-byte tile scales must not be streamed (146 us).  128 lanes x 2 runs per
// workgroup: 256 x 2 111.4, 512 x 2 112.1, 128 x 4 117, 256 x 4 119, 1024 x 1 129 us (one load in flight per lane
// is not enough when the nibbles come from memory).
constexpr int DEQUANT_THREADS = 128;
constexpr int DEQUANT_UNROLL = 2;

// E4M3 magnitude byte of e2m1(code) * 2^(6-d) for d in [12, 19], rounded to nearest-even.
// e2m1(code) = h/2 with h below; in units of the E4M3 subnormal quantum 2^-9 the value is
// h * 2^(14-d).
struct UnderflowTable {
    uint32_t lo[8], hi[8];
};

constexpr uint32_t e4m3_code_of_quanta(uint32_t n) // n quanta of 2^-9, n exactly representable
{
    if (n < 16)
        return n; // subnormals and the first binade share the spacing of one quantum
    uint32_t e = 1;
    while (n >= 16) { // normalise to 8..15 quanta * 2^(e-1)
        n >>= 1;
        ++e;
    }
    return (e << 3) | (n - 8);
}

constexpr uint32_t underflow_entry(int d, int code)
{
    constexpr uint32_t h[8] = {0, 1, 2, 3, 4, 6, 8, 12};
    if (d <= 14)
        return e4m3_code_of_quanta(h[code] << (14 - d));
    const int sh = d - 14;
    if (sh > 8)
        return 0;
    const uint32_t q = h[code] >> sh, rem = h[code] & ((1u << sh) - 1u), half = 1u << (sh - 1);
    return q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u);
}

constexpr UnderflowTable make_underflow_table()
{
    UnderflowTable t{};
    for (int i = 0; i < 8; ++i) {
        const int d = 12 + i;
        t.lo[i] = underflow_entry(d, 0) | underflow_entry(d, 1) << 8 | underflow_entry(d, 2) << 16 |
                  underflow_entry(d, 3) << 24;
        t.hi[i] = underflow_entry(d, 4) | underflow_entry(d, 5) << 8 | underflow_entry(d, 6) << 16 |
                  underflow_entry(d, 7) << 24;
    }
    return t;
}

__constant__ UnderflowTable c_underflow = make_underflow_table();
static_assert(make_underflow_table().lo[0] == 0x0c080400u && make_underflow_table().hi[0] == 0x1c181410u,
              "d = 12 row");
static_assert(make_underflow_table().lo[7] == 0 && make_underflow_table().hi[7] == 0, "d = 19 row is zero");

// One half-block: 16 packed nibbles (two dwords) and their block's scale byte -> 16 E4M3 bytes.  The 8 lanes of
// a 128-element tile call it together (lanes 2j, 2j+1 hold block j) and agree on the tile maximum by DPP.
// Returns the tile's maximum non-NaN scale byte and whether any of its four bytes is NaN.
__device__ __forceinline__ u32x4 dequant_half_block(const u32x2 w, const uint32_t b, uint32_t *tile_max, uint32_t *tile_nan)
{
    // max over the tile's non-NaN scale bytes, and whether any of them is NaN.  Mirroring the 8 lanes pairs
    // block j with block 3-j, swapping quad halves pairs the two results.
    const uint32_t is_nan = b == 255u ? 1u : 0u;
    uint32_t bmax = is_nan ? 0u : b;
    uint32_t any_nan = is_nan;
    bmax = max(bmax, dpp_read<DPP_ROW_HALF_MIRROR>(bmax));
    any_nan |= dpp_read<DPP_ROW_HALF_MIRROR>(any_nan);
    bmax = max(bmax, dpp_read<DPP_QUAD_XOR2>(bmax));
    any_nan |= dpp_read<DPP_QUAD_XOR2>(any_nan);

    // the block's 8-entry table: magnitude code -> E4M3 magnitude byte
    const uint32_t d = bmax - (is_nan ? bmax : b);
    uint32_t t_lo, t_hi;
    if (d <= 11u) {
        t_lo = 0x6c686000u - d * 0x08080800u; // 0, 2^5, 2^6, 1.5*2^6 in E4M3, minus d binades
        t_hi = 0x7c787470u - d * 0x08080808u; // 2^7, 1.5*2^7, 2^8, 1.5*2^8
    } else {
        const uint32_t i = min(d - 12u, 7u);
        t_lo = c_underflow.lo[i];
        t_hi = c_underflow.hi[i];
    }
    uint32_t sign_even = 0x08080808u, sign_odd = 0x80808080u;
    if (is_nan) { // a NaN scale byte: the block's 32 outputs are the E4M3 NaN 0x7F
        t_lo = t_hi = 0x7f7f7f7fu;
        sign_even = sign_odd = 0u;
    }

    u32x4 o;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t wj = w[j];
        const uint32_t mag_even = perm(t_hi, t_lo, wj & 0x07070707u);
        const uint32_t mag_odd = perm(t_hi, t_lo, (wj >> 4) & 0x07070707u);
        const uint32_t even = mag_even | ((wj & sign_even) << 4);
        const uint32_t odd = mag_odd | (wj & sign_odd);
        o[2 * j] = perm(odd, even, 0x05010400u);     // elements 0..3 of this dword
        o[2 * j + 1] = perm(odd, even, 0x07030602u); // elements 4..7
    }
    *tile_max = bmax;
    *tile_nan = any_nan;
    return o;
}

// FP32 tile scale 2^(bmax - 6 - 127): the byte goes straight into the FP32 exponent field; below exponent
// field 1 the same power of two is an FP32 subnormal.
__device__ __forceinline__ float tile_scale_of(uint32_t bmax, uint32_t any_nan)
{
    const int b8 = (int)bmax - 6;
    uint32_t bits = b8 >= 1 ? (uint32_t)b8 << 23 : 0x00400000u >> (uint32_t)(-b8);
    bits = any_nan ? 0x7fc00000u : bits;
    return u2f(bits);
}

struct DequantArgs {
    const uint8_t *q;
    const uint8_t *sf;
    uint8_t *x;
    float *x_scale;
    int64_t ld_q;
    int64_t ld_sf;
    uint32_t n_halves;      // M * K / 16
    uint32_t halves_per_row; // K / 16
};

// One workgroup covers DEQUANT_UNROLL runs of DEQUANT_THREADS consecutive half-blocks; a lane takes
// half-block `tid` of each run: 512 B loaded and 1 KiB stored per wave instruction, both
// contiguous, which is what lets the stores go out non-temporally at full rate.
template <bool DENSE>
__global__ void __launch_bounds__(DEQUANT_THREADS) dequant_to_fp8_kernel(const DequantArgs a)
{
    const uint32_t c0 = blockIdx.x * (DEQUANT_THREADS * DEQUANT_UNROLL) + threadIdx.x;

    u32x2 w[DEQUANT_UNROLL];
    uint32_t sfb[DEQUANT_UNROLL];
#pragma unroll
    for (int u = 0; u < DEQUANT_UNROLL; ++u) {
        const uint32_t c = c0 + u * DEQUANT_THREADS;
        if (c >= a.n_halves)
            break; // n_halves is a multiple of 8: the 8 lanes of a tile leave together
        const uint8_t *src;
        const uint8_t *src_sf;
        if (DENSE) {
            src = a.q + (size_t)c * 8;
            src_sf = a.sf + (c >> 1);
        } else {
            const uint32_t row = c / a.halves_per_row;
            const uint32_t ch = c - row * a.halves_per_row;
            src = a.q + (size_t)row * a.ld_q + (size_t)ch * 8;
            src_sf = a.sf + (size_t)row * a.ld_sf + (ch >> 1);
        }
        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(src));
        sfb[u] = *src_sf;
    }

#pragma unroll
    for (int u = 0; u < DEQUANT_UNROLL; ++u) {
        const uint32_t c = c0 + u * DEQUANT_THREADS;
        if (c >= a.n_halves)
            break;
        uint32_t bmax, any_nan;
        const u32x4 o = dequant_half_block(w[u], sfb[u], &bmax, &any_nan);
        store_streaming(a.x + (size_t)c * 16, o);

        if ((threadIdx.x & 7u) == 0u)
            a.x_scale[c >> 3] = tile_scale_of(bmax, any_nan);
    }
}

// Row-strided inputs (per-token records of nibbles then scale bytes) go through the same kernel with the row
// index divided out per lane.  Measured and not built: a workgroup fetching 1, 2, 4 or 8 whole rows with 16-byte
// loads into LDS and converting from there (262144 records of 3808 bytes: 500-644 us against 488 us) -- the
// load / barrier / convert phases of such a workgroup overlap worse than this kernel's independent lanes.
hipError_t launch_dequant_to_fp8(const uint8_t *q, int64_t ld_q, const uint8_t *sf, int64_t ld_sf,
                                 int64_t M, int64_t K, uint8_t *x, float *x_scale, hipStream_t stream)
{
    DequantArgs a;
    a.q = q;
    a.sf = sf;
    a.x = x;
    a.x_scale = x_scale;
    a.ld_q = ld_q;
    a.ld_sf = ld_sf;
    a.n_halves = (uint32_t)(M * (K / 16));
    a.halves_per_row = (uint32_t)(K / 16);
    constexpr uint32_t per_block = DEQUANT_THREADS * DEQUANT_UNROLL;
    const uint32_t blocks = (a.n_halves + per_block - 1) / per_block;
    const bool dense = ld_q == K / 2 && ld_sf == K / 32;
    if (dense)
        hipLaunchKernelGGL(dequant_to_fp8_kernel<true>, dim3(blocks), dim3(DEQUANT_THREADS), 0, stream, a);
    else
        hipLaunchKernelGGL(dequant_to_fp8_kernel<false>, dim3(blocks), dim3(DEQUANT_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
