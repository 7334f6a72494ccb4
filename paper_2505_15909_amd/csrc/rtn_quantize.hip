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
//   q      clamp( rint( fp32_ieee_div(w, S) ) ) -- w and S have 11-bit significands, so the
//          exact quotient is either an exact tie (representable, returned exactly by an IEEE
//          division) or at least 2^-13 away from one; fp32 rounding cannot move it across.
//          A reciprocal-multiply would not have this property and is not used.
#include "rtn_device.h"
#include "rtn_internal.h"

namespace rtn {

template <int BITS>
__device__ __forceinline__ int quantize_one(float w, float s) {
    float r = rintf(w / s);                              // v_rndne_f32: ties to even
    r = fminf(fmaxf(r, (float)Layout<BITS>::QMIN), (float)Layout<BITS>::QMAX);
    int q = (int)r;
    return (s == 0.0f) ? 0 : q;                           // all-zero / underflowed scale
}

// 8 consecutive-k halves (one 16-byte load) -> 8 codes, offset binary, in layout order.
// 4-bit: one word.  8-bit: two words.
template <int BITS>
__device__ __forceinline__ void quantize_octet(const u32x4_t& raw, float s, uint32_t* out) {
    Half8Words h;
    h.v = __builtin_bit_cast(half8_t, raw);
    if constexpr (BITS == 4) {
        constexpr int NIB[8] = {0, 4, 1, 5, 2, 6, 3, 7};
        uint32_t word = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int q = quantize_one<4>((float)h.v[e], s);
            word |= (uint32_t)(q + 8) << (4 * NIB[e]);
        }
        out[0] = word;
    } else {
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w0 |= (uint32_t)(quantize_one<8>((float)h.v[e], s) + 128) << (8 * e);
            w1 |= (uint32_t)(quantize_one<8>((float)h.v[e + 4], s) + 128) << (8 * e);
        }
        out[0] = w0;
        out[1] = w1;
    }
}

__device__ __forceinline__ float octet_amax(const u32x4_t& raw, float m) {
    half8_t v = __builtin_bit_cast(half8_t, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf((float)v[e]));
    return m;
}

__device__ __forceinline__ float scale_from_amax(float amax, float divisor) {
    return (float)(half_t)(amax / divisor);               // IEEE divide, then fp16 RNE
}

// ---------------------------------------------------------------------------------------
// Small groups (g = TPG tiles, TPG in {1, 2, 4}): one wavefront owns a (row-tile, group)
// unit, keeps its 16 x g block in registers, reduces amax across the four lanes that share a
// row, and quantises from registers: W is read exactly once.
// ---------------------------------------------------------------------------------------
template <int BITS, int TPG>
__global__ __launch_bounds__(256) void quantize_small_group_kernel(
    const half_t* __restrict__ W, uint8_t* __restrict__ qweight, half_t* __restrict__ scales,
    int64_t N, int64_t K, int64_t units, float divisor) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int OPT = TK / 32;                          // octets (16-byte loads) per lane per tile
    const int lane = threadIdx.x & 63;
    const int nl = lane & 15, kq = lane >> 4;
    const int64_t G = K / (TPG * TK);                     // groups per row
    const int64_t KT = K / TK;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t u = wave0; u < units; u += nwaves) {
        const int64_t nt = u / G, j = u % G;
        const half_t* src = W + (nt * 16 + nl) * K + j * (TPG * TK) + kq * 8;
        u32x4_t raw[TPG][OPT];
#pragma unroll
        for (int tp = 0; tp < TPG; ++tp)
#pragma unroll
            for (int t = 0; t < OPT; ++t)
                raw[tp][t] = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
        float m = 0.0f;
#pragma unroll
        for (int tp = 0; tp < TPG; ++tp)
#pragma unroll
            for (int t = 0; t < OPT; ++t) m = octet_amax(raw[tp][t], m);
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        const float s = scale_from_amax(m, divisor);
        if (kq == 0) scales[(nt * 16 + nl) * G + j] = (half_t)s;
        uint8_t* dst = qweight + ((nt * KT + j * TPG) * 64 + lane) * 16;
#pragma unroll
        for (int tp = 0; tp < TPG; ++tp) {
            u32x4_t chunk;
            uint32_t words[4];
#pragma unroll
            for (int t = 0; t < OPT; ++t) quantize_octet<BITS>(raw[tp][t], s, &words[t * (4 / OPT)]);
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

    float m = 0.0f;
    for (int64_t tp = wave; tp < TPG; tp += nwave) {
#pragma unroll
        for (int t = 0; t < OPT; ++t)
            m = octet_amax(*reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32), m);
    }
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    if (kq == 0) row_max[wave][nl] = m;
    __syncthreads();
    m = 0.0f;
    for (int w = 0; w < nwave; ++w) m = fmaxf(m, row_max[w][nl]);
    const float s = scale_from_amax(m, divisor);
    if (wave == 0 && kq == 0) scales[(nt * 16 + nl) * G + j] = (half_t)s;

    uint8_t* dst = qweight + ((nt * KT + j * TPG) * 64 + lane) * 16;
    for (int64_t tp = wave; tp < TPG; tp += nwave) {
        u32x4_t chunk;
        uint32_t words[4];
#pragma unroll
        for (int t = 0; t < OPT; ++t) {
            u32x4_t raw = *reinterpret_cast<const u32x4_t*>(src + tp * TK + t * 32);
            quantize_octet<BITS>(raw, s, &words[t * (4 / OPT)]);
        }
        chunk[0] = words[0]; chunk[1] = words[1]; chunk[2] = words[2]; chunk[3] = words[3];
        *reinterpret_cast<u32x4_t*>(dst + tp * 1024) = chunk;
    }
}

// ---------------------------------------------------------------------------------------
// Inverse of the layout: packed -> int8 codes [N, K] (test hook) or -> fp16 q * S [N, K]
// (dequantise-to-16-bit, first half of the large-input path of Section 5).
// One thread per 16-byte chunk.
// ---------------------------------------------------------------------------------------
template <int BITS, bool DEQUANT>
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ qweight,
                                                     const half_t* __restrict__ scales, void* __restrict__ out,
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
            half8_t o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (half_t)((float)v[e] * (float)s);
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

template <int BITS>
static hipError_t launch_quantize_bits(const void* W, int64_t N, int64_t K, int64_t g, float divisor,
                                       void* qweight, void* scales, hipStream_t st) {
    constexpr int TK = Layout<BITS>::TK;
    const half_t* w = static_cast<const half_t*>(W);
    uint8_t* q = static_cast<uint8_t*>(qweight);
    half_t* s = static_cast<half_t*>(scales);
    const int64_t tpg = g / TK;
    const int64_t units = (N / 16) * (K / g);
    if (tpg == 1 || tpg == 2 || tpg == 4) {
        int64_t blocks = (units + 3) / 4;
        if (blocks > 256 * 64) blocks = 256 * 64;             // grid-stride beyond this
        dim3 grid((unsigned)blocks), block(256);
        if (tpg == 1) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 1>), grid, block, 0, st, w, q, s, N, K, units, divisor);
        else if (tpg == 2) hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 2>), grid, block, 0, st, w, q, s, N, K, units, divisor);
        else hipLaunchKernelGGL((quantize_small_group_kernel<BITS, 4>), grid, block, 0, st, w, q, s, N, K, units, divisor);
    } else {
        // enough wavefronts to cover the group, at most 16
        int waves = (int)(tpg < 16 ? tpg : 16);
        dim3 grid((unsigned)units), block(64 * waves);
        hipLaunchKernelGGL((quantize_large_group_kernel<BITS>), grid, block, 0, st, w, q, s, N, K, g, divisor);
    }
    return hipGetLastError();
}

hipError_t launch_quantize(const void* W, int64_t N, int64_t K, int bits, int64_t g, float divisor,
                           void* qweight, void* scales, hipStream_t st) {
    return bits == 4 ? launch_quantize_bits<4>(W, N, K, g, divisor, qweight, scales, st)
                     : launch_quantize_bits<8>(W, N, K, g, divisor, qweight, scales, st);
}

hipError_t launch_unpack(const void* qweight, const void* scales, int64_t N, int64_t K, int bits, int64_t g,
                         bool dequant, void* out, hipStream_t st) {
    const int64_t chunks = N * K * bits / 8 / 16;
    dim3 grid((unsigned)((chunks + 255) / 256)), block(256);
    const uint8_t* q = static_cast<const uint8_t*>(qweight);
    const half_t* s = static_cast<const half_t*>(scales);
    if (bits == 4) {
        if (dequant) hipLaunchKernelGGL((unpack_kernel<4, true>), grid, block, 0, st, q, s, out, N, K, g);
        else hipLaunchKernelGGL((unpack_kernel<4, false>), grid, block, 0, st, q, s, out, N, K, g);
    } else {
        if (dequant) hipLaunchKernelGGL((unpack_kernel<8, true>), grid, block, 0, st, q, s, out, N, K, g);
        else hipLaunchKernelGGL((unpack_kernel<8, false>), grid, block, 0, st, q, s, out, N, K, g);
    }
    return hipGetLastError();
}

}  // namespace rtn
