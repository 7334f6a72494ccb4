// Fused dequantise-GEMM for larger batches (Section 5: the same weight-only quantised linear layer,
// C = A (q S)^T, when more than a few tokens are processed at once and the matrix cores, not the weight
// stream, start to bound the time).
//
// Wide MFMA kernel.  A workgroup is WV (4, 8 or 16) wavefronts side by side along N that share the staged
// activations -- the wider the workgroup, the fewer times the activations cross from L2 to a compute unit,
// which is what bounds this kernel once a few dozen rows are in play; every wavefront owns NBW
// consecutive 16-row weight tile-rows (16 NBW output columns) and all 16 MB activation rows of the
// workgroup's row block, i.e. a (16 MB) x (16 NBW) register tile of fp32 accumulators:
//   - packed weights go from global memory straight into registers in MFMA operand order (that is what
//     the packed layout is for), three 128-column k-steps deep, and are unpacked once per k-step for all
//     MB row blocks;
//   - the activations of a k-step (16 MB rows x 128 columns) are staged through LDS by the whole
//     workgroup, double buffered, in 16-byte pieces whose position inside a row is XOR-swizzled with
//     the row number so that both the staging writes and the b128 operand reads are conflict-free
//     without padding; one operand read feeds NBW MFMAs;
//   - arithmetic is that of the skinny kernel: exact integer codes into v_mfma_f32_16x16x32_f16, the
//     fp16 scale applied in fp32 to the partial sum of each group (or of the part of a group that lies
//     in this workgroup's k-range: scaling is linear, so groups may straddle split-K boundaries).
// Row blocks of 16 MB rows beyond the first are separate workgroups that re-read the weights; the
// workgroup index is decoded so that the workgroups sharing a weight range are dispatched back to back on
// the same XCD and the second reader hits that XCD's L2.
#include "rtn_device.h"
#include "rtn_internal.h"

namespace rtn {

namespace {

constexpr int kStepK = 128;                     // columns per k-step
constexpr uint32_t kOutOfRange = 0x7FFF0000u;   // beyond any resource size used here (< 2 GiB)
constexpr int kBufferFlags = 0x00020000;        // raw buffer, 32-bit data format
constexpr int kXcds = 8;

struct WideParams {
    const half_t* A;
    const uint8_t* qw;
    const half_t* scales;
    const half_t* zeros;   // asymmetric variant only (ZP)
    half_t* C;
    float* ws;
    int M, N, K;
    int G;              // groups per row
    int spg;            // k-steps per group (g / 128)
    int NT;             // N / 16
    int KL;             // tiles per weight row
    int KS;             // k-steps per row (K / 128)
    int XB;             // workgroups along N
    int ZB;             // row blocks
    int split_k;
    int ks_base, ks_rem;   // workgroup sg covers k-steps [sg*ks_base + min(sg, ks_rem), ...)
    uint32_t spg_inv;      // floor(2^32 / spg) + 1 (0 when spg == 1): k-step -> group by multiply-high
    uint32_t qw_bytes, sc_bytes, a_bytes;
};

// G1: one k-step per group (group size 128): every k-step starts its partial sums from zero, which the
// first MFMA of the step takes as a constant operand instead of a cleared register.
// At least two wavefronts per SIMD (256 registers each): the MFMAs then keep their accumulators in ordinary
// vector registers, where the scale multiply-add can read them directly.
// ZP: asymmetric variant -- the integer zero point of the step's group goes into the unpack (operand = q + Z).
// PS: the weights are scaled in fp16 on their way into the MFMA (fp16(q S), one rounding per weight, as in the tile
// kernel) instead of the group's partial sums in fp32: no second accumulator set, which is what lets a wavefront own
// 128 rows (MB = 8: every unpacked operand feeds 8 MFMAs, and 4 scale multiplies replace 32 multiply-adds).
template <int BITS, int MB, int NBW, bool G1, int WV, bool ZP = false, bool PS = false>
__global__ __launch_bounds__(64 * WV, WV <= 8 ? 2 : 4) void wide_mfma_kernel(const WideParams p) {
    constexpr int TK = Layout<BITS>::TK;
    constexpr int MPT = Layout<BITS>::MFMA_PER_TILE;
    constexpr int TPS = kStepK / TK;                      // tiles per k-step and tile-row: 1 / 2
    constexpr int ROWS = 16 * MB;
    constexpr int BUF_BYTES = ROWS * kStepK * 2;
    __shared__ __align__(16) uint8_t lds_a[2 * BUF_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nl = lane & 15, kq = lane >> 4;

    // workgroup index -> (N block, row block): the ZB row blocks of one N block are kXcds apart
    const int L = blockIdx.x;
    const int xcd = L % kXcds, idx = L / kXcds;
    const int z = idx % p.ZB;
    const int xb = (idx / p.ZB) * kXcds + xcd;
    if (xb >= p.XB) return;                               // padding of the last group of 8 (whole workgroup)
    const int m0 = z * ROWS;
    const int sg = blockIdx.y;
    const int ks0 = sg * p.ks_base + min(sg, p.ks_rem);
    const int T = p.ks_base + (sg < p.ks_rem ? 1 : 0);    // k-steps of this workgroup

    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.qw), 0, p.qw_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p.scales), 0, p.sc_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p.A), 0, p.a_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(ZP ? p.zeros : p.scales), 0, p.sc_bytes, kBufferFlags);
    (void)rz;
    const uint32_t magic = fp16_magic_vgpr();

    const int nt0 = (xb * WV + wave) * NBW;               // first tile-row of this wavefront
    // Load addresses: the lane's part goes into the vector offset, fixed for the whole kernel (out of range once and
    // for all for tile-rows and activation rows that do not exist); the k-step's part is wave-uniform and goes into the
    // scalar offset, so a step's loads cost no vector instructions.  Prefetches past the workgroup's last step load
    // that last step again (in bounds, never used).
    uint32_t w_lane[NBW], s_lane[NBW];
    bool nt_ok[NBW];
#pragma unroll
    for (int r = 0; r < NBW; ++r) {
        nt_ok[r] = nt0 + r < p.NT;
        w_lane[r] = nt_ok[r] ? (uint32_t)(nt0 + r) * (uint32_t)p.KL * 1024u + lane * 16 : kOutOfRange;
        s_lane[r] = nt_ok[r] ? ((uint32_t)(nt0 + r) * 16 + nl) * (uint32_t)p.G * 2u : kOutOfRange;
    }

    // ---- activation staging: thread t moves the 16-byte piece st_p of rows st_row0, st_row0 + RP, ... ----
    constexpr int RP = 4 * WV;                            // rows covered by one pass of the workgroup's threads
    constexpr int NP = (ROWS + RP - 1) / RP;              // passes
    const int st_p = tid & 15, st_row0 = tid >> 4;        // row & 15 == st_row0 & 15 in every pass
    u32x4_t areg[NP];
    uint32_t a_lane[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int row = st_row0 + RP * i;
        a_lane[i] = (row < ROWS && m0 + row < p.M) ? ((uint32_t)(m0 + row) * (uint32_t)p.K + st_p * 8) * 2u : kOutOfRange;
    }
    auto a_load = [&](int t) {                            // k-step t of this workgroup (rows that do not exist: zeros)
        const int so = (int)((uint32_t)(ks0 + min(t, T - 1)) * (kStepK * 2u));
#pragma unroll
        for (int i = 0; i < NP; ++i) areg[i] = __builtin_amdgcn_raw_buffer_load_b128(ra, a_lane[i], so, 0);
    };
    auto a_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int row = st_row0 + RP * i;
            if (ROWS % RP == 0 || row < ROWS)
                *reinterpret_cast<u32x4_t*>(lds_a + buf * BUF_BYTES + (row * 16 + (st_p ^ (row & 15))) * 16) = areg[i];
        }
    };

    // ---- weight / scale ring, three k-steps deep ----
    u32x4_t wbuf[3][NBW][TPS];
    uint16_t sbuf[3][NBW];
    uint16_t zbuf[ZP ? 3 : 1][NBW];                        // zero points, same offsets as the scales
    (void)zbuf;
    auto w_load = [&](int slot, int t) {
        const uint32_t ks = (uint32_t)(ks0 + min(t, T - 1));
        const uint32_t j = (G1 || p.spg_inv == 0) ? ks : __umulhi(ks, p.spg_inv);
#pragma unroll
        for (int r = 0; r < NBW; ++r) {
            sbuf[slot][r] = __builtin_amdgcn_raw_buffer_load_b16(rs, s_lane[r], (int)(j * 2u), 0);
            if constexpr (ZP) zbuf[slot][r] = __builtin_amdgcn_raw_buffer_load_b16(rz, s_lane[r], (int)(j * 2u), 0);
#pragma unroll
            for (int c = 0; c < TPS; ++c)
                wbuf[slot][r][c] = __builtin_amdgcn_raw_buffer_load_b128(rw, w_lane[r], (int)((ks * TPS + c) * 1024u), 2 /* nt */);
        }
    };

    constexpr int NPART = PS ? 1 : MB;                    // no per-group partial sums when the weights are pre-scaled
    float4_t acc[MB][NBW], part[NPART][NBW];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int r = 0; r < NBW; ++r) {
            acc[b][r] = (float4_t){0.f, 0.f, 0.f, 0.f};
            if (b < NPART) part[b][r] = (float4_t){0.f, 0.f, 0.f, 0.f};
        }

    auto scale_row = [&](int slot, int r) {
        if constexpr (!PS) {
            const float sc = (float)__builtin_bit_cast(half_t, sbuf[slot][r]);
#pragma unroll
            for (int b = 0; b < MB; ++b) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[b][r][e] = fmaf(sc, part[b][r][e], acc[b][r][e]);
                if constexpr (!G1) part[b][r] = (float4_t){0.f, 0.f, 0.f, 0.f};
            }
        }
    };

    // steps left in the current group when this workgroup starts
    int left = p.spg - (int)((uint32_t)ks0 - (p.spg_inv == 0 ? (uint32_t)ks0 : __umulhi((uint32_t)ks0, p.spg_inv)) * (uint32_t)p.spg);

    auto step = [&](int slot, int t) {
        a_store((t + 1) & 1);                             // A(t+1), loaded during the previous step
        a_load(t + 2);
        w_load((slot + 2) % 3, t + 2);
        __builtin_amdgcn_sched_barrier(0);                // keep the prefetch ahead of this step's arithmetic
        const uint8_t* abase = lds_a + (t & 1) * BUF_BYTES + (nl * 16) * 16;
        if constexpr (PS) {
            // pre-scaled weights: a 32-column slice is NBW scaled operands against the row blocks, four blocks at a time
            constexpr int HB = MB > 4 ? 4 : MB, NH = MB / HB;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                half8_t bw[NBW];
#pragma unroll
                for (int r = 0; r < NBW; ++r) {
                    Half8Words h;
                    h.v = unpack_operand<BITS>(wbuf[slot][r][i / MPT], i % MPT, magic);
                    const half_t sh = __builtin_bit_cast(half_t, sbuf[slot][r]);
                    const half2_t s2 = {sh, sh};
#pragma unroll
                    for (int e = 0; e < 4; ++e) h.h2[e] = h.h2[e] * s2;
                    bw[r] = h.v;
                }
#pragma unroll
                for (int hb = 0; hb < NH; ++hb) {
                    half8_t a[HB];
#pragma unroll
                    for (int b = 0; b < HB; ++b)
                        a[b] = *reinterpret_cast<const half8_t*>(abase + ((hb * HB + b) * 256 + ((i * 4 + kq) ^ nl)) * 16);
#pragma unroll
                    for (int r = 0; r < NBW; ++r)
#pragma unroll
                        for (int b = 0; b < HB; ++b)
                            acc[hb * HB + b][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[b], bw[r], acc[hb * HB + b][r], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __syncthreads();
            return;
        }
        // the group, or this workgroup's share of it, ends with this step
        const bool ends = G1 ? true : ((--left == 0) || (t == T - 1));
        // the activation operands of a 32-column slice are read one slice ahead of the MFMAs that use them
        half8_t a_next[MB];
#pragma unroll
        for (int b = 0; b < MB; ++b) a_next[b] = *reinterpret_cast<const half8_t*>(abase + (b * 256 + (kq ^ nl)) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half8_t a[MB];
#pragma unroll
            for (int b = 0; b < MB; ++b) a[b] = a_next[b];
            if (i < 3) {
#pragma unroll
                for (int b = 0; b < MB; ++b)
                    a_next[b] = *reinterpret_cast<const half8_t*>(abase + (b * 256 + (((i + 1) * 4 + kq) ^ nl)) * 16);
            }
#pragma unroll
            for (int r = 0; r < NBW; ++r) {
                half8_t bw;
                if constexpr (ZP) bw = unpack_operand_zp<BITS>(wbuf[slot][r][i / MPT], i % MPT, magic, (float)__builtin_bit_cast(half_t, zbuf[slot][r]));
                else bw = unpack_operand<BITS>(wbuf[slot][r][i / MPT], i % MPT, magic);
#pragma unroll
                for (int b = 0; b < MB; ++b) {
                    const float4_t c_in = (G1 && i == 0) ? (float4_t){0.f, 0.f, 0.f, 0.f} : part[b][r];
                    part[b][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[b], bw, c_in, 0, 0, 0);
                }
                if (i == 3 && ends && r > 0) scale_row(slot, r - 1);     // overlaps the next tile-row's MFMAs
            }
            if (i < 3) __builtin_amdgcn_sched_barrier(0);                // keeps the next slice's reads ahead of this slice's MFMAs
        }
        if (ends) {
            scale_row(slot, NBW - 1);
            left = p.spg;
        }
        __syncthreads();
    };

    // ---- prologue: the same issue order as in the loop (activations of a step before its weights), so that
    // the loop's waits are counted waits and not waits for everything ----
    a_load(0);
    w_load(0, 0);
    a_store(0);
    a_load(1);
    w_load(1, 1);
    __syncthreads();

    int t = 0;
    for (; t + 3 <= T; t += 3) {          // no control flow between steps: every wait inside is an exact count
        step(0, t);
        step(1, t + 1);
        step(2, t + 2);
    }
    if (t < T) {
        step(0, t);
        if (t + 1 < T) step(1, t + 1);
    }

    // ---- store: lane holds rows m = 16 b + 4 kq + e, column n = 16 (nt0 + r) + nl ----
#pragma unroll
    for (int r = 0; r < NBW; ++r) {
        if (!nt_ok[r]) continue;
        const int n = (nt0 + r) * 16 + nl;
#pragma unroll
        for (int b = 0; b < MB; ++b) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = m0 + b * 16 + kq * 4 + e;
                if (m < p.M) {
                    if (p.split_k == 1) p.C[(int64_t)m * p.N + n] = (half_t)acc[b][r][e];
                    else p.ws[((int64_t)sg * p.M + m) * p.N + n] = acc[b][r][e];
                }
            }
        }
    }
}

template <int BITS, int MB, int NBW, int WV>
hipError_t launch_wide_g1(const WideParams& wp, dim3 grid, hipStream_t st) {
    dim3 block(64 * WV);
    if (wp.spg == 1) hipLaunchKernelGGL((wide_mfma_kernel<BITS, MB, NBW, true, WV>), grid, block, 0, st, wp);
    else hipLaunchKernelGGL((wide_mfma_kernel<BITS, MB, NBW, false, WV>), grid, block, 0, st, wp);
    return hipGetLastError();
}

// Asymmetric variant: 8 wavefronts, one or two tile-rows per wavefront.
template <int BITS, int MB, int NBW>
hipError_t launch_wide_zp(const WideParams& wp, dim3 grid, hipStream_t st) {
    dim3 block(64 * 8);
    if (wp.spg == 1) hipLaunchKernelGGL((wide_mfma_kernel<BITS, MB, NBW, true, 8, true>), grid, block, 0, st, wp);
    else hipLaunchKernelGGL((wide_mfma_kernel<BITS, MB, NBW, false, 8, true>), grid, block, 0, st, wp);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_wide_zp_bits(const WideParams& wp, int mb, int nbw, dim3 grid, hipStream_t st) {
    switch (mb * 10 + nbw) {
        case 21: return launch_wide_zp<BITS, 2, 1>(wp, grid, st);
        case 22: return launch_wide_zp<BITS, 2, 2>(wp, grid, st);
        case 31: return launch_wide_zp<BITS, 3, 1>(wp, grid, st);
        case 32: return launch_wide_zp<BITS, 3, 2>(wp, grid, st);
        case 41: return launch_wide_zp<BITS, 4, 1>(wp, grid, st);
        case 42: return launch_wide_zp<BITS, 4, 2>(wp, grid, st);
        default: return hipErrorInvalidValue;
    }
}

// Sixteen wavefronts leave 128 registers each: only the register tiles with one tile-row per wavefront.
template <int BITS, int MB, int NBW>
hipError_t launch_wide_wv(const WideParams& wp, int wv, dim3 grid, hipStream_t st) {
    if (wv == 4) return launch_wide_g1<BITS, MB, NBW, 4>(wp, grid, st);
    if (wv == 8) return launch_wide_g1<BITS, MB, NBW, 8>(wp, grid, st);
    if constexpr (NBW == 1) {
        if (wv == 16) return launch_wide_g1<BITS, MB, NBW, 16>(wp, grid, st);
    }
    return hipErrorInvalidValue;
}

// Register tiles of up to 8 accumulator blocks (MB * NBW <= 8) fit 256 registers without spilling; the 128 x 32 tile
// (16 blocks) does with pre-scaled weights, which need no second accumulator set.
template <int BITS>
hipError_t launch_wide_bits(const WideParams& wp, int mb, int nbw, int wv, dim3 grid, hipStream_t st) {
    if (mb == 8) {
        if (nbw != 2 || wv != 8) return hipErrorInvalidValue;
        if (wp.spg == 1) hipLaunchKernelGGL((wide_mfma_kernel<BITS, 8, 2, true, 8, false, true>), grid, dim3(64 * 8), 0, st, wp);
        else hipLaunchKernelGGL((wide_mfma_kernel<BITS, 8, 2, false, 8, false, true>), grid, dim3(64 * 8), 0, st, wp);
        return hipGetLastError();
    }
    switch (mb * 10 + nbw) {
        case 21: return launch_wide_wv<BITS, 2, 1>(wp, wv, grid, st);
        case 22: return launch_wide_wv<BITS, 2, 2>(wp, wv, grid, st);
        case 24: return launch_wide_wv<BITS, 2, 4>(wp, wv, grid, st);
        case 31: return launch_wide_wv<BITS, 3, 1>(wp, wv, grid, st);
        case 32: return launch_wide_wv<BITS, 3, 2>(wp, wv, grid, st);
        case 41: return launch_wide_wv<BITS, 4, 1>(wp, wv, grid, st);
        case 42: return launch_wide_wv<BITS, 4, 2>(wp, wv, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool wide_plan_valid(const LinearArgs& a, const LinearPlan& p) {
    if (a.g % kStepK != 0) return false;
    if (p.m_rows16 == 8) {                                // 128 x 32 register tile, pre-scaled weights
        return !a.zeros && p.n_tiles16 == 2 && p.waves_n == 8 && p.split_k >= 1 && p.split_k <= a.K / kStepK;
    }
    if (p.m_rows16 < 2 || p.m_rows16 > 4) return false;
    if (p.n_tiles16 != 1 && p.n_tiles16 != 2 && p.n_tiles16 != 4) return false;
    if (p.m_rows16 * p.n_tiles16 > 8) return false;       // register tile: at most 8 accumulator blocks
    if (p.waves_n != 4 && p.waves_n != 8 && !(p.waves_n == 16 && p.n_tiles16 == 1)) return false;
    if (p.split_k < 1 || p.split_k > a.K / kStepK) return false;
    if (a.zeros && (p.waves_n != 8 || p.n_tiles16 > 2)) return false;      // the zero-point instantiations
    return true;
}

hipError_t launch_linear_wide(const LinearArgs& a, const LinearPlan& p, hipStream_t st) {
    const int tk = (a.bits == 4) ? 128 : 64;
    WideParams wp;
    wp.A = static_cast<const half_t*>(a.A);
    wp.qw = static_cast<const uint8_t*>(a.qweight);
    wp.scales = static_cast<const half_t*>(a.scales);
    wp.zeros = static_cast<const half_t*>(a.zeros);
    wp.C = static_cast<half_t*>(a.C);
    wp.ws = a.workspace;
    wp.M = (int)a.M; wp.N = (int)a.N; wp.K = (int)a.K;
    wp.G = (int)(a.K / a.g);
    wp.spg = (int)(a.g / kStepK);
    wp.spg_inv = wp.spg == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint32_t)wp.spg) + 1u;
    wp.NT = (int)(a.N / 16);
    wp.KL = (int)(a.K / tk);
    wp.KS = (int)(a.K / kStepK);
    const int cols_wg = 16 * p.n_tiles16 * p.waves_n;
    wp.XB = (int)((a.N + cols_wg - 1) / cols_wg);
    wp.ZB = p.m_blocks;
    wp.split_k = p.split_k;
    wp.ks_base = wp.KS / p.split_k;
    wp.ks_rem = wp.KS % p.split_k;
    wp.qw_bytes = (uint32_t)((size_t)a.N * a.K * a.bits / 8);
    wp.sc_bytes = (uint32_t)((size_t)a.N * wp.G * 2);
    wp.a_bytes = (uint32_t)((size_t)a.M * a.K * 2);
    const int xb_pad = (wp.XB + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(xb_pad * wp.ZB), (unsigned)p.split_k, 1);
    hipError_t e;
    if (a.zeros) e = (a.bits == 4) ? launch_wide_zp_bits<4>(wp, p.m_rows16, p.n_tiles16, grid, st)
                                   : launch_wide_zp_bits<8>(wp, p.m_rows16, p.n_tiles16, grid, st);
    else e = (a.bits == 4) ? launch_wide_bits<4>(wp, p.m_rows16, p.n_tiles16, p.waves_n, grid, st)
                           : launch_wide_bits<8>(wp, p.m_rows16, p.n_tiles16, p.waves_n, grid, st);
    if (e != hipSuccess) return e;
    if (p.split_k > 1) e = launch_splitk_reduce(a.workspace, static_cast<half_t*>(a.C), a.M * a.N, p.split_k, st);
    return e;
}

}  // namespace rtn
