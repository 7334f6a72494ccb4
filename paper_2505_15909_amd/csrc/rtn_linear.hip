// Fused dequantise-GEMM of the RTN weight-only quantised linear layer for gfx950
// (Sections 2.3 and 5: 16-bit activations times 4-/8-bit weights at token-generation batch
// sizes, where every weight byte is used once and time = weight bytes / HBM bandwidth).
//
//   C[m, n] = fp16( sum_k A[m, k] * q[n, k] * S[n, k / g] )
//
// Skinny MFMA kernel.  A wavefront owns R weight tiles-rows (16 output channels each) and a
// slice of K.  Per step it streams one k-chunk (4 tiles = 4 KiB, four 16-byte-per-lane loads,
// issued one step ahead) of one tile-row, unpacks the codes in registers to exact fp16
// integers, and feeds them as the B operand of v_mfma_f32_16x16x32_f16; the A operand is the
// (zero-padded to 16 rows) activation block, staged once per workgroup in LDS (double
// buffered, padded rows -> conflict-free 16-byte reads) and held in registers across the R
// tile-rows.  Scales multiply the fp32 partial sum of each group (exact codes into the matrix
// cores, one fp32 multiply-add per group and output), never the individual weights.
// Wavefronts of a workgroup are arranged WN along N (sharing the staged activations) times WK
// along K (in-workgroup split-K, reduced through LDS in a fixed order); an optional global
// split-K writes fp32 partials to the workspace and a second kernel sums them in a fixed
// order, so results are bit-reproducible.
//
// MFMA operand maps (16x16x32 f16): a-operand lane l = row l % 16, k-slot l / 16 (8 halves);
// b-operand lane l = column l % 16, same k-slot; result lane l, register e = row 4 (l/16) + e,
// column l % 16.  Rows are batch entries m, columns are output channels n, so every lane needs
// exactly one scale per group (that of its own weight row).
#include "rtn_device.h"
#include "rtn_internal.h"

namespace rtn {

constexpr int kChunkTiles = 4;       // tiles (16-byte loads per lane) per k-chunk
constexpr int kStagePieces = 4;      // 16-byte pieces of activations a thread stages per stage
constexpr int kLdsPadHalves = 8;     // row padding: row stride = 16 bytes mod 256 bytes

struct SkinnyParams {
    const half_t* A;
    const uint8_t* qw;
    const half_t* scales;
    half_t* C;
    float* ws;
    int M, N, K;
    int G;            // groups per row
    int g;            // group size
    int NT;           // N / 16
    int KL;           // tiles per row
    int KC;           // chunks per row
    int WN, WK, wn_shift;   // wave = wk * WN + wn
    int wk_shift;
    int split_k;
    int lds_rows;     // activation rows staged (min(M, 16))
};

template <int BITS>
struct Geom {
    static constexpr int TK = Layout<BITS>::TK;
    static constexpr int MPT = Layout<BITS>::MFMA_PER_TILE;
    static constexpr int CK = kChunkTiles * TK;           // k per chunk: 512 / 256
    static constexpr int NM = kChunkTiles * MPT;          // MFMAs per chunk: 16 / 8
    static constexpr int CK8_SHIFT = (BITS == 4) ? 6 : 5; // log2(CK / 8)
};

template <int NGC>
struct ScaleVec;
template <> struct ScaleVec<1> { typedef uint16_t raw_t; };
template <> struct ScaleVec<2> { typedef uint32_t raw_t; };
template <> struct ScaleVec<4> { typedef u32x2_t raw_t; };

template <int NGC>
__device__ __forceinline__ float scale_at(const typename ScaleVec<NGC>::raw_t& raw, int i) {
    if constexpr (NGC == 1) {
        return (float)__builtin_bit_cast(half_t, raw);
    } else if constexpr (NGC == 2) {
        half2_t h = __builtin_bit_cast(half2_t, raw);
        return (float)h[i];
    } else {
        const uint32_t word = raw[i >> 1];     // by value: bit_cast of a vector-element lvalue reads element 0
        half2_t h = __builtin_bit_cast(half2_t, word);
        return (float)h[i & 1];
    }
}

template <int BITS, int R, int NGC>
__global__ __launch_bounds__(512) void skinny_mfma_kernel(const SkinnyParams p) {
    typedef Geom<BITS> GM;
    typedef typename ScaleVec<NGC>::raw_t sraw_t;
    extern __shared__ __align__(16) uint8_t lds_bytes[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wn = wave & (p.WN - 1), wk = wave >> p.wn_shift;
    const int nl = lane & 15, kq = lane >> 4;
    const int nthreads = blockDim.x;

    const int m0 = blockIdx.z * 16;
    const int Mb = min(16, p.M - m0);
    const half_t* __restrict__ A = p.A + (int64_t)m0 * p.K;

    const int sg = blockIdx.y;
    const int cb0 = (int)((int64_t)p.KC * sg / p.split_k);
    const int cb1 = (int)((int64_t)p.KC * (sg + 1) / p.split_k);
    const int nstage = (cb1 - cb0 + p.WK - 1) >> p.wk_shift;
    const int KS = p.WK * GM::CK;
    const int ks8_shift = GM::CK8_SHIFT + p.wk_shift;      // log2(KS / 8)
    const int lds_stride = KS + kLdsPadHalves;             // halves
    half_t* lds_a = reinterpret_cast<half_t*>(lds_bytes);
    const int lds_buf = p.lds_rows * lds_stride;           // halves per buffer

    // tile-rows of this wavefront (clamped for loads, masked for stores)
    const int ntile0 = (blockIdx.x * p.WN + wn) * R;
    const uint8_t* wbase[R];
    const half_t* sbase[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = min(ntile0 + r, p.NT - 1);
        wbase[r] = p.qw + ((int64_t)nt * p.KL) * 1024 + lane * 16;
        sbase[r] = p.scales + ((int64_t)nt * 16 + nl) * p.G;
    }

    // ---- staging helpers -------------------------------------------------------------
    u32x4_t stg[kStagePieces];
    auto stage_fetch = [&](int s) {
        const int kbase = (cb0 + s * p.WK) * GM::CK;
        const int klimit = cb1 * GM::CK;
        const int total = Mb << ks8_shift;
#pragma unroll
        for (int i = 0; i < kStagePieces; ++i) {
            const int idx = tid + i * nthreads;
            const int m = idx >> ks8_shift, o = idx & ((1 << ks8_shift) - 1);
            const int k = kbase + o * 8;
            if (idx < total && k < klimit)
                stg[i] = *reinterpret_cast<const u32x4_t*>(A + (int64_t)m * p.K + k);
        }
    };
    auto stage_commit = [&](int s) {
        const int kbase = (cb0 + s * p.WK) * GM::CK;
        const int klimit = cb1 * GM::CK;
        const int total = Mb << ks8_shift;
        half_t* dst = lds_a + (s & 1) * lds_buf;
#pragma unroll
        for (int i = 0; i < kStagePieces; ++i) {
            const int idx = tid + i * nthreads;
            const int m = idx >> ks8_shift, o = idx & ((1 << ks8_shift) - 1);
            const int k = kbase + o * 8;
            if (idx < total && k < klimit)
                *reinterpret_cast<u32x4_t*>(dst + m * lds_stride + o * 8) = stg[i];
        }
    };

    // ---- weight / scale prefetch -----------------------------------------------------
    auto scale_index = [&](int ci) -> int64_t {
        // first group of chunk ci: ci * CK / g
        return (NGC > 1) ? (int64_t)ci * NGC : ((int64_t)ci * GM::CK) / p.g;
    };
    auto fetch_w = [&](int r, int ci, u32x4_t (&wv)[kChunkTiles], sraw_t& sv) {
        const uint8_t* src = wbase[r] + (int64_t)ci * (kChunkTiles * 1024);
#pragma unroll
        for (int c = 0; c < kChunkTiles; ++c) wv[c] = load_stream16(src + c * 1024);
        sv = *reinterpret_cast<const sraw_t*>(sbase[r] + scale_index(ci));
    };

    float4_t acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = (float4_t){0.f, 0.f, 0.f, 0.f};

    u32x4_t wnext[kChunkTiles];
    sraw_t snext;
    int ci = cb0 + wk;                                     // this wavefront's chunk in stage 0
    if (ci < cb1) fetch_w(0, ci, wnext, snext);            // in flight while activations are staged
    stage_fetch(0);
    stage_commit(0);
    __syncthreads();

    for (int s = 0; s < nstage; ++s) {
        const bool more = (s + 1 < nstage);
        if (more) stage_fetch(s + 1);
        const bool valid = ci < cb1;
        half8_t areg[GM::NM];
        if (valid) {
            const half_t* src = lds_a + (s & 1) * lds_buf + nl * lds_stride + wk * GM::CK + kq * 8;
#pragma unroll
            for (int i = 0; i < GM::NM; ++i) {
                if (nl < Mb) areg[i] = *reinterpret_cast<const half8_t*>(src + i * 32);
                else areg[i] = (half8_t){0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            u32x4_t wcur[kChunkTiles];
            sraw_t scur = snext;
#pragma unroll
            for (int c = 0; c < kChunkTiles; ++c) wcur[c] = wnext[c];
            // issue the next step's loads before computing this one
            if (r + 1 < R) {
                if (valid) fetch_w(r + 1, ci, wnext, snext);
            } else {
                if (ci + p.WK < cb1) fetch_w(0, ci + p.WK, wnext, snext);
            }
            if (valid) {
                constexpr int TPGRP = kChunkTiles / NGC;   // tiles per group inside a chunk
#pragma unroll
                for (int gi = 0; gi < NGC; ++gi) {
                    float4_t part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = gi * TPGRP; c < (gi + 1) * TPGRP; ++c) {
#pragma unroll
                        for (int t = 0; t < GM::MPT; ++t) {
                            const half8_t b = unpack_operand<BITS>(wcur[c], t);
                            part = __builtin_amdgcn_mfma_f32_16x16x32_f16(areg[c * GM::MPT + t], b, part, 0, 0, 0);
                        }
                    }
                    const float sc = scale_at<NGC>(scur, gi);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][e] = fmaf(sc, part[e], acc[r][e]);
                }
            }
        }
        if (more) stage_commit(s + 1);
        __syncthreads();
        ci += p.WK;
    }

    // ---- in-workgroup split-K reduction (fixed order) ----------------------------------
    if (p.WK > 1) {
        float4_t* red = reinterpret_cast<float4_t*>(lds_bytes);
        if (wk > 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) red[(((wk - 1) * p.WN + wn) * R + r) * 64 + lane] = acc[r];
        }
        __syncthreads();
        if (wk == 0) {
            for (int w = 1; w < p.WK; ++w) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const float4_t v = red[(((w - 1) * p.WN + wn) * R + r) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][e] += v[e];
                }
            }
        }
    }
    if (wk != 0) return;

    // ---- store: lane holds rows m = 4 kq + e, column n = 16 tile + nl --------------------
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int nt = ntile0 + r;
        if (nt >= p.NT) continue;
        const int n = nt * 16 + nl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = kq * 4 + e;
            if (m < Mb) {
                if (p.split_k == 1) p.C[(int64_t)(m0 + m) * p.N + n] = (half_t)acc[r][e];
                else p.ws[((int64_t)sg * p.M + (m0 + m)) * p.N + n] = acc[r][e];
            }
        }
    }
}

// Sums the split-K partials in a fixed order and rounds once to fp16.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ ws, half_t* __restrict__ C,
                                                            int64_t MN, int split_k) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= MN) return;
    if (i + 4 <= MN) {
        float4_t v = *reinterpret_cast<const float4_t*>(ws + i);
        for (int s = 1; s < split_k; ++s) {
            const float4_t u = *reinterpret_cast<const float4_t*>(ws + (int64_t)s * MN + i);
            v += u;
        }
        typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
        half4_t h = {(half_t)v[0], (half_t)v[1], (half_t)v[2], (half_t)v[3]};
        *reinterpret_cast<half4_t*>(C + i) = h;
    } else {
        for (int64_t j = i; j < MN; ++j) {
            float v = ws[j];
            for (int s = 1; s < split_k; ++s) v += ws[(int64_t)s * MN + j];
            C[j] = (half_t)v;
        }
    }
}

static int ilog2(int v) {
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

size_t linear_lds_bytes(const LinearArgs& a, const LinearPlan& p) {
    const int ck = (a.bits == 4) ? 512 : 256;
    const int rows = (int)(a.M < 16 ? a.M : 16);
    const size_t stage = (size_t)2 * rows * (p.waves_k * ck + kLdsPadHalves) * 2;
    const size_t red = p.waves_k > 1 ? (size_t)(p.waves_k - 1) * p.waves_n * p.r_tiles * 1024 : 0;
    return stage > red ? stage : red;
}

template <int BITS, int R>
static hipError_t launch_skinny_ngc(const SkinnyParams& sp, int ngc, dim3 grid, dim3 block, size_t lds,
                                    hipStream_t st) {
    switch (ngc) {
        case 1: hipLaunchKernelGGL((skinny_mfma_kernel<BITS, R, 1>), grid, block, lds, st, sp); break;
        case 2: hipLaunchKernelGGL((skinny_mfma_kernel<BITS, R, 2>), grid, block, lds, st, sp); break;
        default: hipLaunchKernelGGL((skinny_mfma_kernel<BITS, R, 4>), grid, block, lds, st, sp); break;
    }
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_skinny_r(const SkinnyParams& sp, int r, int ngc, dim3 grid, dim3 block, size_t lds,
                                  hipStream_t st) {
    switch (r) {
        case 1: return launch_skinny_ngc<BITS, 1>(sp, ngc, grid, block, lds, st);
        case 2: return launch_skinny_ngc<BITS, 2>(sp, ngc, grid, block, lds, st);
        default: return launch_skinny_ngc<BITS, 4>(sp, ngc, grid, block, lds, st);
    }
}

hipError_t launch_linear(const LinearArgs& a, const LinearPlan& p, hipStream_t st) {
    const int tk = (a.bits == 4) ? 128 : 64;
    const int ck = kChunkTiles * tk;
    SkinnyParams sp;
    sp.A = static_cast<const half_t*>(a.A);
    sp.qw = static_cast<const uint8_t*>(a.qweight);
    sp.scales = static_cast<const half_t*>(a.scales);
    sp.C = static_cast<half_t*>(a.C);
    sp.ws = a.workspace;
    sp.M = (int)a.M; sp.N = (int)a.N; sp.K = (int)a.K;
    sp.g = (int)a.g;
    sp.G = (int)(a.K / a.g);
    sp.NT = (int)(a.N / 16);
    sp.KL = (int)(a.K / tk);
    sp.KC = (int)(a.K / ck);
    sp.WN = p.waves_n; sp.WK = p.waves_k;
    sp.wn_shift = ilog2(p.waves_n);
    sp.wk_shift = ilog2(p.waves_k);
    sp.split_k = p.split_k;
    sp.lds_rows = (int)(a.M < 16 ? a.M : 16);
    const int ngc = (a.g >= ck) ? 1 : (int)(ck / a.g);
    const int rows_per_block = p.waves_n * p.r_tiles;
    dim3 grid((unsigned)((sp.NT + rows_per_block - 1) / rows_per_block), (unsigned)p.split_k, (unsigned)p.m_blocks);
    dim3 block((unsigned)(64 * p.waves_n * p.waves_k));
    const size_t lds = linear_lds_bytes(a, p);
    hipError_t e = (a.bits == 4) ? launch_skinny_r<4>(sp, p.r_tiles, ngc, grid, block, lds, st)
                                 : launch_skinny_r<8>(sp, p.r_tiles, ngc, grid, block, lds, st);
    if (e != hipSuccess) return e;
    if (p.split_k > 1) {
        const int64_t MN = a.M * a.N;
        dim3 rgrid((unsigned)((MN / 4 + 255) / 256 + 1)), rblock(256);
        hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, rblock, 0, st, a.workspace, sp.C, MN, p.split_k);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace rtn
