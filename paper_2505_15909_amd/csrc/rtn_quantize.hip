// Load-time RTN quantise-and-pack for gfx950 (Section 2.2, Eq. 1 and Eq. 2; Section 5: the
// quantised weights are reshuffled once into the layout the GEMM kernel expects).
//
// Both kernels read fp16 W [N, K] row-major and write the packed tiles and the fp16 scales
// [N, K/g].  A wavefront produces one 1 KiB tile per store instruction (16 bytes per lane,
// fully coalesced).  Lane l of a tile owns row l % 16 and the columns 32 t + 8 (l / 16) + e.
//
// Arithmetic (bit-exact by construction, no fast-math anywhere in this file):
//   amax   exact (max of |fp16| values, held in fp32)
//   S      fp16_rne( fp32_ieee_div(amax, D) )   -- equal to the single rounding of the exact
//          quotient for every fp16 amax and D in {7, 127, 7.5, 127.5}
//   q      clamp( rint( w / S ) ) without a per-element division: with r = fp32_ieee_div(1, S), shared by
//          the group, and the even constant C = 768 + B (B = 8 or 128, the offset of the stored code),
//              y = fma(w, r, C)      one fp32 rounding of the exact w r + C, which lies in [512, 2048),
//                                    where fp32 values are the multiples of 2^-14 (2^-13 from 1024 up,
//                                    reached only under subnormal S, where |Q| can approach 1.5 D)
//              z = rint(y)           ties to even
//              stored code = clamp(z, C + QMIN, C + QMAX) - 768
//          Why z - C is the round-half-even of the exact quotient Q = w / S.  w and S carry 11-bit
//          significands, so Q is either exactly a half-integer h or at least 1/4094 > 2^-13 away from every
//          half-integer (2w - (2i+1)S is a non-zero multiple of the smaller of their quanta).  The exact
//          product P = w r satisfies |P - Q| <= |Q| 2^-24 < 2^-16 (|Q| < 192 inside a group).
//          (a) Q = h is a tie: h + C is a grid point and |P + C - (h + C)| < 2^-16 is less than half a
//              grid step (>= 2^-15), so the fma returns h + C exactly and rint applies ties-to-even to
//              the true tie; C is even, so the parity of the result is that of the code.
//          (b) Q is not a tie: for every half-integer h, |P - h| > 2^-13 - 2^-16 > 2^-14, at least half
//              a grid step, so the fma cannot round onto h + C and, rounding being monotone, y stays
//              strictly on Q's side of it: rint(y) = rint(Q) + C.
//          The first rounding (to the 2^-14 grid) and the second (to integers) are both needed: adding a
//          constant with unit ulp directly would misround true ties by the error of P.
//          S == 0 (all-zero or underflowed group): r is forced to 0, y = C, the code is 0.
//          The clamp matters for the Eq. 2 divisor and for subnormal S, whose rounding is coarse.
//   pack   the integers z are < 1024, so sums  z_a + 16 z_b + 256 z_c + 4096 z_d  (4-bit) and
//          z_a + 256 z_b (8-bit) are exact in fp32; they are formed by fma, converted once, joined
//          with a shift-add, and the constant contributed by the 768s is subtracted from the word.
#include "rtn_device.h"
#include "rtn_internal.h"

namespace rtn {

template <int BITS>
__device__ __forceinline__ float snapped_code(half_t w, float r) {
    constexpr float C = 768.0f + (BITS == 4 ? 8.0f : 128.0f);
    const float y = fmaf((float)w, r, C);                // v_fma_mix_f32: the fp16 operand converts exactly
    return __builtin_amdgcn_fmed3f(rintf(y), C + (float)Layout<BITS>::QMIN, C + (float)Layout<BITS>::QMAX);
}

__device__ __forceinline__ float group_reciprocal(float s) { return s == 0.0f ? 0.0f : 1.0f / s; }   // IEEE divide

// 8 consecutive-k halves (one 16-byte load) -> 8 codes, offset binary, in layout order.
// 4-bit: one word.  8-bit: two words.
template <int BITS>
__device__ __forceinline__ void quantize_octet(const u32x4_t& raw, float r, uint32_t* out) {
    Half8Words h;
    h.v = __builtin_bit_cast(half8_t, raw);
    float z[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = snapped_code<BITS>(h.v[e], r);
    if constexpr (BITS == 4) {
        // element e sits in nibble {0,4,1,5,2,6,3,7}[e]: even elements fill the low half-word
        const float lo = fmaf(z[6], 4096.0f, fmaf(z[4], 256.0f, fmaf(z[2], 16.0f, z[0])));
        const float hi = fmaf(z[7], 4096.0f, fmaf(z[5], 256.0f, fmaf(z[3], 16.0f, z[1])));
        out[0] = (((uint32_t)hi << 16) + (uint32_t)lo) - 0x33333300u;      // 768 * 0x1111 in both halves
    } else {
        const float a = fmaf(z[1], 256.0f, z[0]), b = fmaf(z[3], 256.0f, z[2]);
        const float c = fmaf(z[5], 256.0f, z[4]), d = fmaf(z[7], 256.0f, z[6]);
        out[0] = (((uint32_t)b << 16) + (uint32_t)a) - 0x03030300u;        // 768 * 0x101 in both halves
        out[1] = (((uint32_t)d << 16) + (uint32_t)c) - 0x03030300u;
    }
}

// Running maximum of |x| over packed fp16 pairs: max3(m, x, -x) per 32-bit word.  For the finite inputs
// the library accepts this is the plain maximum; it stays in fp16, where it is exact.
__device__ __forceinline__ uint32_t pk_amax(uint32_t m, uint32_t x) {
    uint32_t o;
    asm("v_pk_maximum3_f16 %0, %1, %2, %2 neg_lo:[0,0,1] neg_hi:[0,0,1]" : "=v"(o) : "v"(m), "v"(x));
    return o;
}

__device__ __forceinline__ uint32_t octet_amax(const u32x4_t& raw, uint32_t m) {
#pragma unroll
    for (int i = 0; i < 4; ++i) m = pk_amax(m, raw[i]);
    return m;
}

__device__ __forceinline__ float amax_of_pair(uint32_t m) {
    const half2_t v = __builtin_bit_cast(half2_t, m);
    return fmaxf((float)v[0], (float)v[1]);
}

__device__ __forceinline__ float scale_from_amax(float amax, float divisor) {
    return (float)(half_t)(amax / divisor);               // IEEE divide, then fp16 RNE
}

// ---------------------------------------------------------------------------------------
// Small groups: one wavefront owns a 16-row block of TPG tiles (TPG in {1, 2, 4}) that holds SUB groups per
// row (SUB = 1: g = TPG tiles; SUB = 2 or 4 with TPG = 1: g = half or a quarter of a tile, down to 32 columns),
// keeps it in registers, reduces amax across the four lanes that share a row, and quantises from registers: W is
// read exactly once.
// ---------------------------------------------------------------------------------------
template <int BITS, int TPG, int SUB>
__global__ __launch_bounds__(256) void quantize_small_group_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    int64_t N, int64_t K, int64_t units, float divisor) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;                          // octets (16-byte loads) per lane per tile
    constexpr int OPS = OPT / SUB;                        // octets per lane per sub-group (SUB > 1 only with TPG == 1)
    static_assert(SUB == 1 || (TPG == 1 && OPT % SUB == 0), "sub-tile groups need one tile per unit");
    const int lane = threadIdx.x & 63;
    const int nl = lane & 15, kq = lane >> 4;
    const int64_t U = K / (TPG * TK);                     // units per row
    const int64_t G = U * SUB;                            // groups per row
    const int64_t KT = K / TK;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t u = wave0; u < units; u += nwaves) {
        const int64_t nt = u / U, j = u % U;
        const half_t* src = W + (nt * 16 + nl) * K + j * (TPG * TK) + kq * 8;
        u32x4_t raw[TPG][OPT];
#pragma unroll
        for (int tp = 0; tp < TPG; ++tp)
#pragma unroll
            for (int t = 0; t < OPT; ++t)
                raw[tp][t] = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
        float r[SUB];
#pragma unroll
        for (int sg = 0; sg < SUB; ++sg) {
            uint32_t m2 = 0u;
            if constexpr (SUB == 1) {
#pragma unroll
                for (int tp = 0; tp < TPG; ++tp)
#pragma unroll
                    for (int t = 0; t < OPT; ++t) m2 = octet_amax(raw[tp][t], m2);
            } else {
#pragma unroll
                for (int t = 0; t < OPS; ++t) m2 = octet_amax(raw[0][sg * OPS + t], m2);
            }
            float m = amax_of_pair(m2);
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            const float s = scale_from_amax(m, divisor);
            r[sg] = group_reciprocal(s);
            if (kq == 0) scales[(nt * 16 + nl) * G + j * SUB + sg] = (half_t)s;
        }
        uint8_t* dst = qweight + ((nt * KT + j * TPG) * 64 + lane) * 16;
#pragma unroll
        for (int tp = 0; tp < TPG; ++tp) {
            u32x4_t chunk;
            uint32_t words[4];
#pragma unroll
            for (int t = 0; t < OPT; ++t) quantize_octet<BITS>(raw[tp][t], r[SUB == 1 ? 0 : t / OPS], &words[t * (4 / OPT)]);
            chunk[0] = words[0]; chunk[1] = words[1]; chunk[2] = words[2]; chunk[3] = words[3];
            *reinterpret_cast<u32x4_t*>(dst + (int64_t)tp * 1024) = chunk;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Large groups, including one group per output channel (g = K): a workgroup owns a
// (row-tile, group) unit.  Pass 1 streams the 16 x g block for the 16 row maxima (reduced
// through LDS), pass 2 streams it again (from L2 / Infinity Cache for all but the largest g)
// and packs.
// ---------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(1024) void quantize_large_group_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    int64_t N, int64_t K, int64_t g, float divisor) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;
    __shared__ float row_max[16][16];                    // [wave][row]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwave = blockDim.x >> 6;
    const int nl = lane & 15, kq = lane >> 4;
    const int64_t G = K / g, KT = K / TK, TPG = g / TK;
    const int64_t u = blockIdx.x;
    const int64_t nt = u / G, j = u % G;
    const half_t* src = W + (nt * 16 + nl) * K + j * g + kq * 8;

    uint32_t m2 = 0u;
    for (int64_t tp = wave; tp < TPG; tp += nwave) {
#pragma unroll
        for (int t = 0; t < OPT; ++t)
            m2 = octet_amax(*reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32), m2);
    }
    float m = amax_of_pair(m2);
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    if (kq == 0) row_max[wave][nl] = m;
    __syncthreads();
    m = 0.0f;
    for (int w = 0; w < nwave; ++w) m = fmaxf(m, row_max[w][nl]);
    const float s = scale_from_amax(m, divisor);
    const float r = group_reciprocal(s);
    if (wave == 0 && kq == 0) scales[(nt * 16 + nl) * G + j] = (half_t)s;

    uint8_t* dst = qweight + ((nt * KT + j * TPG) * 64 + lane) * 16;
    for (int64_t tp = wave; tp < TPG; tp += nwave) {
        u32x4_t chunk;
        uint32_t words[4];
#pragma unroll
        for (int t = 0; t < OPT; ++t) {
            u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
            quantize_octet<BITS>(raw, r, &words[t * (4 / OPT)]);
        }
        chunk[0] = words[0]; chunk[1] = words[1]; chunk[2] = words[2]; chunk[3] = words[3];
        *reinterpret_cast<u32x4_t*>(dst + tp * 1024) = chunk;
    }
}

// ---------------------------------------------------------------------------------------
// Medium and wide groups (the per-channel case): a workgroup of NW wavefronts owns ROWS rows of a (row-tile, group)
// unit and keeps that ROWS x g block in registers between the amax pass and the packing pass (LPL 16-byte loads
// per lane, NW KiB x LPL per workgroup), so W is read exactly once.  Blocks of up to 8 loads per lane: 16 wavefronts,
// all 16 rows.  Larger blocks, g up to 14336 or 28672: 8 wavefronts and 8 or 4 rows (two or four workgroups per
// row-tile, each writing its 128- or 64-byte runs of every tile), so that two or three workgroups share a compute
// unit and one loads while another packs and stores -- a single 16-wavefront workgroup per compute unit alternates
// between the two (measured on the 70B and 405B shapes: 4.1-6.4 TB/s against 3.3-5.1).  g up to 57344: 16 wavefronts
// and 4 rows (8 wavefronts would leave 32-byte runs, which halves the rate).
// A wavefront covers 16 / ROWS consecutive tiles per step (lane -> row nl % ROWS of tile nl / ROWS); tiles past the
// end of the group are neither loaded nor stored.
// ---------------------------------------------------------------------------------------
template <int BITS, int LPL, int ROWS, int NW = 16>
__global__ __launch_bounds__(64 * NW) void quantize_resident_group_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    int64_t N, int64_t K, int64_t g, float divisor) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;
    constexpr int TPW = LPL / OPT;                        // steps per wavefront
    constexpr int TPS = 16 / ROWS;                        // tiles per wavefront per step, row blocks per row-tile
    __shared__ float row_max[NW][ROWS];                   // [wave][row]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nl = lane & 15, kq = lane >> 4;
    const int rl = nl % ROWS, sub = nl / ROWS;
    const int64_t G = K / g, KT = K / TK;
    const int TPG = (int)(g / TK);
    const int64_t u = blockIdx.x / TPS;
    const int hb = (int)(blockIdx.x % TPS);               // which ROWS-row block of the row-tile
    const int64_t nt = u / G, j = u % G;
    const int64_t row = nt * 16 + hb * ROWS + rl;
    const half_t* src = W + row * K + j * g + kq * 8;

    u32x4_t raw[TPW][OPT];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tp = (wave + NW * i) * TPS + sub;
#pragma unroll
        for (int t = 0; t < OPT; ++t) {
            raw[i][t] = u32x4_t{0u, 0u, 0u, 0u};
            if (tp < TPG) raw[i][t] = *reinterpret_cast<const u32x4_t*>(src + (int64_t)tp * TK + t * 32);
        }
    }
    uint32_t m2 = 0u;
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int t = 0; t < OPT; ++t) m2 = octet_amax(raw[i][t], m2);
    float m = amax_of_pair(m2);
    m = fmaxf(m, __shfl_xor(m, 16));                      // the four k-quarters of a tile
    m = fmaxf(m, __shfl_xor(m, 32));
    if constexpr (ROWS <= 8) m = fmaxf(m, __shfl_xor(m, 8));    // the tiles of this step that hold the same row
    if constexpr (ROWS <= 4) m = fmaxf(m, __shfl_xor(m, 4));
    if (kq == 0 && sub == 0) row_max[wave][rl] = m;
    __syncthreads();
    m = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) m = fmaxf(m, row_max[w][rl]);
    const float s = scale_from_amax(m, divisor);
    const float r = group_reciprocal(s);
    if (wave == 0 && kq == 0 && sub == 0) scales[row * G + j] = (half_t)s;

    uint8_t* dst = qweight + ((nt * KT + j * TPG) * 64 + kq * 16 + hb * ROWS + rl) * 16;
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tp = (wave + NW * i) * TPS + sub;
        u32x4_t chunk;
        uint32_t words[4];
#pragma unroll
        for (int t = 0; t < OPT; ++t) quantize_octet<BITS>(raw[i][t], r, &words[t * (4 / OPT)]);
        chunk[0] = words[0]; chunk[1] = words[1]; chunk[2] = words[2]; chunk[3] = words[3];
        if (tp < TPG) *reinterpret_cast<u32x4_t*>(dst + (int64_t)tp * 1024) = chunk;
    }
}

// ---------------------------------------------------------------------------------------
// Inverse of the layout: packed -> int8 codes [N, K] (test hook) or -> fp16 q * S [N, K]
// (dequantise-to-16-bit, first half of the large-input path of Section 5).
// One thread per 16-byte chunk.
// ---------------------------------------------------------------------------------------
template <int BITS, bool DEQUANT>
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ qweight,
                                                     const half_t* __restrict__ scales,
                                                     const half_t* __restrict__ zeros, void* __restrict__ out,
                                                     int64_t N, int64_t K, int64_t g) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int MPT = Layout<BITS>::MFMA_PER_TILE;
    const int64_t chunk_id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t KT = K / TK;
    if (chunk_id >= (N / 16) * KT * 64) return;
    const int lane = (int)(chunk_id & 63);
    const int64_t tile = chunk_id >> 6;
    const int64_t nt = tile / KT, kt = tile % KT;
    const int nl = lane & 15, kq = lane >> 4;
    const u32x4_t chunk = *reinterpret_cast<const u32x4_t*>(qweight + chunk_id * 16);
    const int64_t n = nt * 16 + nl;
    const uint32_t magic = fp16_magic_vgpr();
#pragma unroll
    for (int i = 0; i < MPT; ++i) {
        const half8_t v = unpack_operand<BITS>(chunk, i, magic);     // exact integers as fp16
        const int64_t k = kt * TK + i * 32 + kq * 8;
        if constexpr (DEQUANT) {
            const half_t s = scales[n * (K / g) + k / g];
            const float z = zeros ? (float)zeros[n * (K / g) + k / g] : 0.0f;     // asymmetric variant: S (q + Z)
            half8_t o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (half_t)(((float)v[e] + z) * (float)s);   // exact sum and product, one rounding
            *reinterpret_cast<half8_t*>(reinterpret_cast<half_t*>(out) + n * K + k) = o;
        } else {
            u32x2_t o = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[0] |= ((uint32_t)(int)(float)v[e] & 0xFFu) << (8 * e);
                o[1] |= ((uint32_t)(int)(float)v[e + 4] & 0xFFu) << (8 * e);
            }
            *reinterpret_cast<u32x2_t*>(reinterpret_cast<int8_t*>(out) + n * K + k) = o;
        }
    }
}

template <int BITS, int ROWS>
static void launch_resident_rows8(int64_t lpl, dim3 grid, hipStream_t st, const half_t* w, uint8_t* q, half_t* s,
                                  int64_t N, int64_t K, int64_t g, float divisor) {
    dim3 block(512);
    if (lpl <= 16) hipLaunchKernelGGL((quantize_resident_group_kernel<BITS, 16, ROWS, 8>), grid, block, 0, st, w, q, s, N, K, g, divisor);
    else hipLaunchKernelGGL((quantize_resident_group_kernel<BITS, 28, ROWS, 8>), grid, block, 0, st, w, q, s, N, K, g, divisor);
}

// rows == 16: 16 wavefronts and at most 8 loads per lane; 8 wavefronts: 8 or 4 rows, 16 or 28 loads per lane;
// 16 wavefronts and 4 rows: 28 loads per lane
template <int BITS>
static void launch_resident(int rows, int nw, int64_t lpl, dim3 grid, hipStream_t st, const half_t* w, uint8_t* q, half_t* s,
                            int64_t N, int64_t K, int64_t g, float divisor) {
    if (rows == 16) hipLaunchKernelGGL((quantize_resident_group_kernel<BITS, 8, 16, 16>), grid, dim3(1024), 0, st, w, q, s, N, K, g, divisor);
    else if (nw == 16) hipLaunchKernelGGL((quantize_resident_group_kernel<BITS, 28, 4, 16>), grid, dim3(1024), 0, st, w, q, s, N, K, g, divisor);
    else if (rows == 8) launch_resident_rows8<BITS, 8>(lpl, grid, st, w, q, s, N, K, g, divisor);
    else launch_resident_rows8<BITS, 4>(lpl, grid, st, w, q, s, N, K, g, divisor);
}

template <int BITS>
static hipError_t launch_quantize_bits(const void* W, int64_t N, int64_t K, int64_t g, float divisor,
                                       void* qweight, void* scales, hipStream_t st) {
    constexpr int TK = Layout<BITS>::TK;
    const half_t* w = static_cast<const half_t*>(W);
    uint8_t* q = static_cast<uint8_t*>(qweight);
    half_t* s = static_cast<half_t*>(scales);
    const int64_t tpg = g / TK;
    const int64_t units = (N / 16) * (K / g);
    if (g < TK) {                                             // 2 or 4 groups per tile (g = 32 or 64)
        const int sub = (int)(TK / g);
        const int64_t tiles = (N / 16) * (K / TK);
        int64_t blocks = (tiles + 3) / 4;
        if (blocks > 256 * 64) blocks = 256 * 64;
        dim3 grid((unsigned)blocks), block(256);
        if (sub == 2) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 1, 2>), grid, block, 0, st, w, q, s, N, K, tiles, divisor);
        else if constexpr (BITS == 4) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 1, 4>), grid, block, 0, st, w, q, s, N, K, tiles, divisor);
        else return hipErrorInvalidValue;
    } else if (tpg == 1 || tpg == 2 || tpg == 4) {
        int64_t blocks = (units + 3) / 4;
        if (blocks > 256 * 64) blocks = 256 * 64;             // grid-stride beyond this
        dim3 grid((unsigned)blocks), block(256);
        if (tpg == 1) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 1, 1>), grid, block, 0, st, w, q, s, N, K, units, divisor);
        else if (tpg == 2) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 2, 1>), grid, block, 0, st, w, q, s, N, K, units, divisor);
        else hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 4, 1>), grid, block, 0, st, w, q, s, N, K, units, divisor);
    } else if (tpg * (TK / 32) <= 8 * 8 * 28) {
        // the unit, or a half, a quarter or an eighth of its rows, fits the registers of one workgroup
        const int64_t octets = tpg * (TK / 32);
        int rows = 16, nw = 16;
        int64_t lpl = ((tpg + 15) / 16) * (TK / 32);          // 16 wavefronts, all 16 rows
        if (lpl > 8) {
            if (octets <= 4 * 8 * 28) {                       // 8 wavefronts, 8 or 4 rows
                rows = octets <= 2 * 8 * 28 ? 8 : 4;
                nw = 8;
            } else {                                          // 16 wavefronts, 4 rows: 64-byte runs at least
                rows = 4;
            }
            lpl = ((tpg + nw * (16 / rows) - 1) / (nw * (16 / rows))) * (TK / 32);
        }
        dim3 grid((unsigned)(units * (16 / rows)));
        launch_resident<BITS>(rows, nw, lpl, grid, st, w, q, s, N, K, g, divisor);
    } else {
        dim3 grid((unsigned)units), block(1024);
        hipLaunchKernelGGL((quantize_large_group_kernel<BITS>), grid, block, 0, st, w, q, s, N, K, g, divisor);
    }
    return hipGetLastError();
}

hipError_t launch_quantize(const void* W, int64_t N, int64_t K, int bits, int64_t g, float divisor,
                           void* qweight, void* scales, hipStream_t st) {
    return bits == 4 ? launch_quantize_bits<4>(W, N, K, g, divisor, qweight, scales, st)
                     : launch_quantize_bits<8>(W, N, K, g, divisor, qweight, scales, st);
}

// ---------------------------------------------------------------------------------------
// Asymmetric variant (the remark after Eq. 1 in Section 2.2: an integer zero point Z is subtracted from the
// result of Int()).  Per group: [alpha, beta] = [min(min w, 0), max(max w, 0)];
//   S = fp16( (beta - alpha) / (2^b - 1) ), the exact quotient rounded once (exact_quotient_fp16 below)
//   T = clamp( rint( fp32_div(alpha, S) ), -(2^b - 1), 0 ),   Z = T + 2^(b-1)   (stored as fp16, an exact integer)
//   stored code u = clamp( rint(w / S) - T, 0, 2^b - 1 )      (= q + 2^(b-1) with q = clamp(rint(w / S) - Z))
// and the dequantised weight is S (q + Z) = S (u + T).  rint(w / S) comes from the same two-step rounding as in the
// symmetric kernels, y = fma(w, r, C), z = rint(y), now with C = 1536 and WITHOUT the zero point inside C: the tie
// rule applies to w / S, and C must stay even.  |w / S| < 384 (2^b - 1 = 255 levels, times up to 1.5 when S is a
// subnormal fp16 and rounds coarsely), so y lies in (1152, 1920), where fp32 values are the multiples of 2^-13;
// |w r - w / S| <= 384 * 2^-24 < 2^-15 is less than half that step and less than the distance (> 2^-13 - 2^-15) of
// any non-tie quotient from a half-integer, so both cases of the argument at the top of this file carry over.
// alpha / S needs no such care: it is one IEEE division per group, its quotient is either exactly a half-integer
// (representable, returned exactly) or further from one than fp32's spacing there.
// The packing sums stay below 2^24 ((1536 + 255) * 4369 < 2^23).
//
// One wavefront per unit.  SUB == 1: a unit is one group of g >= TK columns of a 16-row tile-row, read twice
// (second pass from cache).  SUB > 1: a unit is one tile holding SUB groups of TK / SUB columns.
// ---------------------------------------------------------------------------------------
struct AsymGroup {
    float r, lo, hi;          // reciprocal scale, clamp bounds C + T and C + T + levels
    uint32_t kconst;          // what the C + T of every code adds to a packed word
};

__device__ __forceinline__ uint32_t pk_min(uint32_t m, uint32_t x) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(half2_t, m), __builtin_bit_cast(half2_t, x)));
}
__device__ __forceinline__ uint32_t pk_max(uint32_t m, uint32_t x) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2_t, m), __builtin_bit_cast(half2_t, x)));
}

// Row-wise (alpha, beta) of a lane's running packed min / max: across the pair, then across the four lanes of a row.
__device__ __forceinline__ void row_range(uint32_t mn2, uint32_t mx2, float* alpha, float* beta) {
    const half2_t a = __builtin_bit_cast(half2_t, mn2), b = __builtin_bit_cast(half2_t, mx2);
    float lo = fminf(fminf((float)a[0], (float)a[1]), 0.0f), hi = fmaxf(fmaxf((float)b[0], (float)b[1]), 0.0f);
    lo = fminf(lo, __shfl_xor(lo, 16));
    hi = fmaxf(hi, __shfl_xor(hi, 16));
    lo = fminf(lo, __shfl_xor(lo, 32));
    hi = fmaxf(hi, __shfl_xor(hi, 32));
    *alpha = lo;
    *beta = hi;
}

// fp16(x / d), the exact quotient rounded once (x = beta - alpha: a difference of two fp16 values, exact in fp64 but
// not in fp32; d = 2^b - 1).  The IEEE fp64 quotient differs from the exact one by at most 2^-53 relative, while an
// exact quotient that is not itself an fp16 midpoint lies at least 2^-42 relative from any (x and midpoint * d are
// both multiples of 2^-25 and x < 2^18), so rounding the fp64 quotient to fp16 equals rounding the exact one.  fp64 ->
// fp16 in one rounding: truncate to fp32 and set the last bit if anything was cut off (round to odd, 24 bits >= 11 +
// 2), then the hardware's fp32 -> fp16 round-to-nearest-even.
__device__ __forceinline__ half_t exact_quotient_fp16(double x, double d) {
    const double q = x / d;                                          // IEEE fp64 division
    float f = __double2float_rz(q);
    if ((double)f != q) f = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, f) | 1u);
    return (half_t)f;
}

template <int BITS>
__device__ __forceinline__ AsymGroup asym_group(float alpha, float beta, half_t* s_out, half_t* z_out) {
    constexpr float LEVELS = (float)((1 << BITS) - 1);
    constexpr float C = 1536.0f;
    const half_t s16 = exact_quotient_fp16((double)beta - (double)alpha, (double)LEVELS);
    const float s = (float)s16;
    float t = (s == 0.0f) ? 0.0f : rintf(alpha / s);                 // IEEE divide
    t = fminf(fmaxf(t, -LEVELS), 0.0f);
    AsymGroup gp;
    gp.r = group_reciprocal(s);
    gp.lo = C + t;
    gp.hi = C + t + LEVELS;
    const uint32_t base = (uint32_t)(C + t);
    gp.kconst = (BITS == 4) ? base * 0x1111u * 0x10001u : base * 0x101u * 0x10001u;     // modulo 2^32
    *s_out = s16;
    *z_out = (half_t)(t + (float)(1 << (BITS - 1)));
    return gp;
}

template <int BITS>
__device__ __forceinline__ void quantize_octet_asym(const u32x4_t& raw, const AsymGroup& gp, uint32_t* out) {
    Half8Words h;
    h.v = __builtin_bit_cast(half8_t, raw);
    float z[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        z[e] = __builtin_amdgcn_fmed3f(rintf(fmaf((float)h.v[e], gp.r, 1536.0f)), gp.lo, gp.hi);
    if constexpr (BITS == 4) {
        const float lo = fmaf(z[6], 4096.0f, fmaf(z[4], 256.0f, fmaf(z[2], 16.0f, z[0])));
        const float hi = fmaf(z[7], 4096.0f, fmaf(z[5], 256.0f, fmaf(z[3], 16.0f, z[1])));
        out[0] = (((uint32_t)hi << 16) + (uint32_t)lo) - gp.kconst;
    } else {
        const float a = fmaf(z[1], 256.0f, z[0]), b = fmaf(z[3], 256.0f, z[2]);
        const float c = fmaf(z[5], 256.0f, z[4]), d = fmaf(z[7], 256.0f, z[6]);
        out[0] = (((uint32_t)b << 16) + (uint32_t)a) - gp.kconst;
        out[1] = (((uint32_t)d << 16) + (uint32_t)c) - gp.kconst;
    }
}

template <int BITS, int SUB>
__global__ __launch_bounds__(256) void quantize_asym_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    half_t* __restrict__ zeros, int64_t N, int64_t K, int64_t g, int64_t units) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;                          // octets (16-byte loads) per lane per tile
    constexpr uint32_t kPosInf = 0x7C007C00u, kNegInf = 0xFC00FC00u;
    const int lane = threadIdx.x & 63;
    const int nl = lane & 15, kq = lane >> 4;
    const int64_t KT = K / TK, G = K / g;
    const int64_t U = (SUB == 1) ? G : KT;                // units per tile-row
    const int tiles = (SUB == 1) ? (int)(g / TK) : 1;     // tiles per unit
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t u = wave0; u < units; u += nwaves) {
        const int64_t nt = u / U, j = u % U;
        const int64_t n = nt * 16 + nl;
        const int64_t kt0 = j * tiles;                    // first tile of the unit
        const half_t* src = W + n * K + kt0 * TK + kq * 8;
        AsymGroup gp[SUB];
        // units of up to kKeep octets per lane (groups of up to 256 codes at 4 bits, 512 at 8 bits) stay in registers between the range pass and the
        // packing pass; larger ones are read again, from cache
        constexpr int kKeep = 8;
        const bool resident = tiles * OPT <= kKeep;
        u32x4_t keep[kKeep];
        if constexpr (SUB == 1) {
            uint32_t mn = kPosInf, mx = kNegInf;
            if (resident) {
#pragma unroll
                for (int t = 0; t < kKeep; ++t) {
                    keep[t] = t < tiles * OPT ? *reinterpret_cast<const u32x4_t*>(src + t * 32) : u32x4_t{0u, 0u, 0u, 0u};
                    if (t < tiles * OPT) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            mn = pk_min(mn, keep[t][i]);
                            mx = pk_max(mx, keep[t][i]);
                        }
                    }
                }
            } else {
                for (int t = 0; t < tiles * OPT; ++t) {
                    const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + t * 32);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        mn = pk_min(mn, raw[i]);
                        mx = pk_max(mx, raw[i]);
                    }
                }
            }
            float alpha, beta;
            row_range(mn, mx, &alpha, &beta);
            half_t s16, z16;
            gp[0] = asym_group<BITS>(alpha, beta, &s16, &z16);
            if (kq == 0) {
                scales[n * G + j] = s16;
                zeros[n * G + j] = z16;
            }
        } else {
            constexpr int OPS = OPT / SUB;                // octets per lane per group
#pragma unroll
            for (int sg = 0; sg < SUB; ++sg) {
                uint32_t mn = kPosInf, mx = kNegInf;
#pragma unroll
                for (int t = 0; t < OPS; ++t) {
                    const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + (sg * OPS + t) * 32);
                    keep[sg * OPS + t] = raw;             // one tile per unit: OPT <= kKeep octets
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        mn = pk_min(mn, raw[i]);
                        mx = pk_max(mx, raw[i]);
                    }
                }
                float alpha, beta;
                row_range(mn, mx, &alpha, &beta);
                half_t s16, z16;
                gp[sg] = asym_group<BITS>(alpha, beta, &s16, &z16);
                if (kq == 0) {
                    scales[n * G + j * SUB + sg] = s16;
                    zeros[n * G + j * SUB + sg] = z16;
                }
            }
        }
        if (resident) {
#pragma unroll
            for (int tp = 0; tp < kKeep / OPT; ++tp) {
                if (tp < tiles) {
                    u32x4_t o;
#pragma unroll
                    for (int t = 0; t < OPT; ++t) {
                        uint32_t wd[BITS == 4 ? 1 : 2];
                        quantize_octet_asym<BITS>(keep[tp * OPT + t], gp[SUB == 1 ? 0 : t / (OPT / SUB)], wd);
                        if constexpr (BITS == 4) o[t] = wd[0];
                        else { o[2 * t] = wd[0]; o[2 * t + 1] = wd[1]; }
                    }
                    *reinterpret_cast<u32x4_t*>(qweight + ((nt * KT + kt0 + tp) * 64 + lane) * 16) = o;
                }
            }
            continue;
        }
        for (int tp = 0; tp < tiles; ++tp) {
            u32x4_t o;
            if constexpr (BITS == 4) {
#pragma unroll
                for (int t = 0; t < OPT; ++t) {
                    const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
                    uint32_t wd[1];
                    quantize_octet_asym<BITS>(raw, gp[SUB == 1 ? 0 : t / (OPT / SUB)], wd);
                    o[t] = wd[0];
                }
            } else {
#pragma unroll
                for (int t = 0; t < OPT; ++t) {
                    const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
                    uint32_t wd[2];
                    quantize_octet_asym<BITS>(raw, gp[SUB == 1 ? 0 : t / (OPT / SUB)], wd);
                    o[2 * t] = wd[0];
                    o[2 * t + 1] = wd[1];
                }
            }
            *reinterpret_cast<u32x4_t*>(qweight + ((nt * KT + kt0 + tp) * 64 + lane) * 16) = o;
        }
    }
}

// Wide groups (per-channel and the like): one 16-wavefront workgroup per (16-row tile-row, group); wavefront w takes the
// tiles w, w + 16, ... of the group, the row ranges meet in LDS, and every wavefront then packs its own tiles (second
// read from cache).
template <int BITS>
__global__ __launch_bounds__(1024) void quantize_asym_wide_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    half_t* __restrict__ zeros, int64_t N, int64_t K, int64_t g) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;
    constexpr uint32_t kPosInf = 0x7C007C00u, kNegInf = 0xFC00FC00u;
    __shared__ float lo_s[16][16], hi_s[16][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nl = lane & 15, kq = lane >> 4;
    const int64_t KT = K / TK, G = K / g;
    const int tiles = (int)(g / TK);
    const int64_t u = blockIdx.x;
    const int64_t nt = u / G, j = u % G;
    const int64_t n = nt * 16 + nl;
    const int64_t kt0 = j * tiles;
    const half_t* src = W + n * K + kt0 * TK + kq * 8;
    uint32_t mn = kPosInf, mx = kNegInf;
    for (int tp = wave; tp < tiles; tp += 16) {
#pragma unroll
        for (int t = 0; t < OPT; ++t) {
            const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                mn = pk_min(mn, raw[i]);
                mx = pk_max(mx, raw[i]);
            }
        }
    }
    float alpha, beta;
    row_range(mn, mx, &alpha, &beta);               // a wavefront without tiles contributes (0, 0), which the range contains anyway
    if (kq == 0) {
        lo_s[wave][nl] = alpha;
        hi_s[wave][nl] = beta;
    }
    __syncthreads();
    alpha = lo_s[0][nl];
    beta = hi_s[0][nl];
#pragma unroll
    for (int w = 1; w < 16; ++w) {
        alpha = fminf(alpha, lo_s[w][nl]);
        beta = fmaxf(beta, hi_s[w][nl]);
    }
    half_t s16, z16;
    const AsymGroup gp = asym_group<BITS>(alpha, beta, &s16, &z16);
    if (wave == 0 && kq == 0) {
        scales[n * G + j] = s16;
        zeros[n * G + j] = z16;
    }
    for (int tp = wave; tp < tiles; tp += 16) {
        u32x4_t o;
#pragma unroll
        for (int t = 0; t < OPT; ++t) {
            const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
            if constexpr (BITS == 4) {
                uint32_t wd[1];
                quantize_octet_asym<BITS>(raw, gp, wd);
                o[t] = wd[0];
            } else {
                uint32_t wd[2];
                quantize_octet_asym<BITS>(raw, gp, wd);
                o[2 * t] = wd[0];
                o[2 * t + 1] = wd[1];
            }
        }
        *reinterpret_cast<u32x4_t*>(qweight + ((nt * KT + kt0 + tp) * 64 + lane) * 16) = o;
    }
}

template <int BITS>
static hipError_t launch_quantize_asym_bits(const void* W, int64_t N, int64_t K, int64_t g, void* qweight, void* scales,
                                            void* zeros, hipStream_t st) {
    constexpr int TK = Layout<BITS>::TK;
    const half_t* w = static_cast<const half_t*>(W);
    uint8_t* q = static_cast<uint8_t*>(qweight);
    half_t* s = static_cast<half_t*>(scales);
    half_t* z = static_cast<half_t*>(zeros);
    const int64_t units = (g < TK) ? (N / 16) * (K / TK) : (N / 16) * (K / g);
    int64_t blocks = (units + 3) / 4;
    if (blocks > 256 * 64) blocks = 256 * 64;             // grid-stride beyond this
    dim3 grid((unsigned)blocks), block(256);
    if (g >= 16 * TK) {                                   // at least one tile per wavefront of a 16-wavefront workgroup
        hipLaunchKernelGGL((quantize_asym_wide_kernel<BITS>), dim3((unsigned)units), dim3(1024), 0, st, w, q, s, z, N, K, g);
    } else if (g >= TK) {
        hipLaunchKernelGGL((quantize_asym_kernel<BITS, 1>), grid, block, 0, st, w, q, s, z, N, K, g, units);
    } else if (TK / g == 2) {
        hipLaunchKernelGGL((quantize_asym_kernel<BITS, 2>), grid, block, 0, st, w, q, s, z, N, K, g, units);
    } else if constexpr (BITS == 4) {
        if (TK / g != 4) return hipErrorInvalidValue;
        hipLaunchKernelGGL((quantize_asym_kernel<BITS, 4>), grid, block, 0, st, w, q, s, z, N, K, g, units);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_quantize_asym(const void* W, int64_t N, int64_t K, int bits, int64_t g, void* qweight, void* scales,
                                void* zeros, hipStream_t st) {
    return bits == 4 ? launch_quantize_asym_bits<4>(W, N, K, g, qweight, scales, zeros, st)
                     : launch_quantize_asym_bits<8>(W, N, K, g, qweight, scales, zeros, st);
}

hipError_t launch_unpack(const void* qweight, const void* scales, int64_t N, int64_t K, int bits, int64_t g,
                         bool dequant, void* out, hipStream_t st, const void* zeros) {
    const int64_t chunks = N * K * bits / 8 / 16;
    dim3 grid((unsigned)((chunks + 255) / 256)), block(256);
    const uint8_t* q = static_cast<const uint8_t*>(qweight);
    const half_t* s = static_cast<const half_t*>(scales);
    const half_t* z = static_cast<const half_t*>(zeros);
    if (bits == 4) {
        if (dequant) hipLaunchKernelGGL((unpack_kernel<4, true>), grid, block, 0, st, q, s, z, out, N, K, g);
        else hipLaunchKernelGGL((unpack_kernel<4, false>), grid, block, 0, st, q, s, z, out, N, K, g);
    } else {
        if (dequant) hipLaunchKernelGGL((unpack_kernel<8, true>), grid, block, 0, st, q, s, z, out, N, K, g);
        else hipLaunchKernelGGL((unpack_kernel<8, false>), grid, block, 0, st, q, s, z, out, N, K, g);
    }
    return hipGetLastError();
}

}  // namespace rtn
