// Matrix-core-bound GEMM of the quantised linear layer for large batches (Section 5: with many input tokens
// the layer is a dense matrix product; the paper then dequantises the weights to 16 bit and calls a dense GEMM,
// and measures where that overtakes the fused kernel).  One kernel core, three weight sources:
//   - packed 4-bit / 8-bit codes: dequantised on the way into LDS (fused path for a hundred rows and more),
//   - dense fp16 weights [N, K]: the 16-bit GEMM of the dequantise-then-GEMM path.
//
// A workgroup of 8 wavefronts (2 along M x 4 along N) computes a TM x 256 tile of C, TM = 128 or 256; a
// wavefront owns (TM / 2) x 64 of it as MBW x 4 v_mfma_f32_16x16x32_f16 blocks (MBW = 4 or 8: 64 or 128 fp32
// accumulator registers).  What bounds a GEMM of this kind on this chip is the traffic from L2 to the compute
// units (about 11 TB/s in aggregate): a TM x 256 x 64 step moves (TM + 256) x 128 bytes of fp16 operands for
// 2 x TM x 256 x 64 flops, 85 flop/B at TM = 128 and 128 flop/B at TM = 256 (packed int4 weights: 175 and
// 210 flop/B), against 64 flop/B for 128 x 128 tiles.
// K advances in steps of 64 columns through two LDS stages (one barrier per step); a row of a staged tile is
// 128 bytes = eight 16-byte pieces, stored at piece ^ (row & 7): conflict-free for the row-wise staging writes, for
// the b128 operand reads (lane -> row nl, piece 4 i + kq) and for the stores of dequantised weights, which have the
// operand pattern (16-byte stores go through 128 bytes per cycle, eight lanes at a time: with piece ^ ((row >> 1) & 7)
// every such store took twice as long, by the bank-conflict counter).  Global loads run two steps
// (activations, dense weights) or one 128-column chunk (packed weights) ahead of their LDS stores, in registers.
//
// Fused dequantisation: a packed tile is unpacked once per workgroup (not once per wavefront), multiplied by
// its group's scale in fp16 (one rounding per weight, relative error 2^-11, far inside the layer's tolerance)
// and written to LDS as ordinary fp16, so the inner loop is that of the dense GEMM and carries no
// per-accumulator scale arithmetic.  The vector ALU and the matrix cores of a SIMD overlap little on this chip
// (measured), so vector instructions per MFMA are what this layout minimises.
#include "rtn_device.h"
#include "rtn_internal.h"

namespace rtn {

namespace {

constexpr int kTN = 256;                        // columns of C per workgroup
constexpr int kBK = 64;                         // columns of K per step
constexpr int kChunkK = 128;                    // packed weights are fetched in 128-column chunks (two steps)
constexpr int kThreads = 512;
constexpr uint32_t kOutOfRange = 0x7FFF0000u;
constexpr int kBufferFlags = 0x00020000;
constexpr int kXcds = 8;

struct TileParams {
    const half_t* A;
    const void* B;          // packed codes or fp16 [N, K]
    const half_t* scales;
    half_t* C;
    float* ws;
    int M, N, K;
    int G;                  // groups per row (packed sources)
    int cpg;                // 128-column chunks per group
    uint32_t cpg_inv;       // floor(2^32 / cpg) + 1 (0 when cpg == 1)
    uint32_t cpg_one;       // all ones when cpg == 1, else 0: chunk -> group is umulhi(c, cpg_inv) + (c & cpg_one)
    int KL;                 // packed tiles per weight row
    int XB, ZB;             // tiles along N, along M
    int split_k;
    int kc_base, kc_rem;    // workgroup sg covers 128-column chunks [sg*kc_base + min(sg, kc_rem), ...)
    uint32_t b_bytes, sc_bytes;   // packed sources only
};

__device__ __forceinline__ uint32_t swizzled(int row, int piece) {      // byte offset inside a staged tile
    return (uint32_t)(row * 128 + ((piece ^ (row & 7)) * 16));
}

// BSRC: 0 = dense fp16 weights, 4 / 8 = packed codes.  MBW: 16-row blocks per wavefront along M (4 or 8).
// PD: prefetch distance of the global loads in steps (activations, dense weights) or chunks (packed weights):
// 2 with the 64-register accumulator tile, 1 with the 128-register one (256 registers per wavefront in all).
template <int BSRC, int MBW, int PD = (MBW == 4 ? 2 : 1)>
__global__ __launch_bounds__(kThreads, 2) void tile_gemm_kernel(const TileParams p) {
    constexpr int TM = 32 * MBW;
    constexpr int A_BYTES = TM * 128, B_BYTES = kTN * 128, STAGE = A_BYTES + B_BYTES;
    extern __shared__ __align__(16) uint8_t lds[];           // two stages: [A tile][B tile]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int nl = lane & 15, kq = lane >> 4;

    // workgroup index -> (N tile, M tile): the ZB row tiles that share a weight tile are dispatched back to
    // back on one XCD
    const int L = blockIdx.x;
    const int xcd = L % kXcds, idx = L / kXcds;
    const int zb = idx % p.ZB;
    const int xb = (idx / p.ZB) * kXcds + xcd;
    if (xb >= p.XB) return;
    const int m0 = zb * TM, n0 = xb * kTN;
    const int sg = blockIdx.y;
    const int kc0 = sg * p.kc_base + min(sg, p.kc_rem);      // first 128-column chunk
    const int T = 2 * (p.kc_base + (sg < p.kc_rem ? 1 : 0)); // 64-column steps of this workgroup
    const int ks0 = 2 * kc0;

    // Row-major fp16 operands are addressed through a resource that starts at this workgroup's first row and
    // ends after its last valid one (rows past M or N read as zeros; no 32-bit limit on the whole matrix).
    const int a_rows = min(TM, p.M - m0), b_rows = min(kTN, p.N - n0);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t*>(p.A) + (int64_t)m0 * p.K, 0, (uint32_t)a_rows * (uint32_t)p.K * 2u, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rb = BSRC == 0
        ? __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(static_cast<const half_t*>(p.B)) + (int64_t)n0 * p.K, 0,
                                            (uint32_t)b_rows * (uint32_t)p.K * 2u, kBufferFlags)
        : __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.B), 0, p.b_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p.scales), 0, p.sc_bytes, kBufferFlags);
    const uint32_t magic = fp16_magic_vgpr();

    // ---- staging of row-major fp16 tiles (A always, B when dense): thread -> piece st_p of rows st_r + 64 i ----
    const int st_p = tid & 7, st_r = tid >> 3;               // (st_r + 64 i) & 7 does not depend on i
    const uint32_t st_off = swizzled(st_r, st_p);            // + i * 64 rows * 128 bytes
    constexpr int NA = TM / 64;                              // pieces per thread per step
    u32x4_t areg[PD][NA];
    auto a_load = [&](int set, int t, int i0 = 0, int i1 = 2 * MBW / 4) {
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            const int row = st_r + 64 * i;
            const bool ok = t < T && row < a_rows;
            const uint32_t off = ok ? ((uint32_t)row * (uint32_t)p.K + (uint32_t)(ks0 + t) * kBK + st_p * 8) * 2u : kOutOfRange;
            areg[set][i] = __builtin_amdgcn_raw_buffer_load_b128(ra, off, 0, 0);
        }
    };
    auto a_store = [&](int set, int stage, int i0 = 0, int i1 = 2 * MBW / 4) {
#pragma unroll
        for (int i = i0; i < i1; ++i) *reinterpret_cast<u32x4_t*>(lds + stage * STAGE + st_off + i * 8192) = areg[set][i];
    };

    // ---- weights ----
    // dense: four pieces per thread per step, two steps ahead (set = step & 1)
    // packed: wavefront w dequantises tile-rows 2w and 2w+1 of the 16 in the weight tile; a 128-column chunk
    // (one int4 tile or two int8 tiles per tile-row, plus its scale) is fetched two chunks ahead (set = chunk & 1)
    constexpr int TPC = BSRC == 8 ? 2 : 1;                   // packed tiles per chunk and tile-row
    constexpr int NBR = BSRC == 0 ? 4 : 2 * TPC;
    u32x4_t breg[PD][NBR];
    uint16_t sreg[PD][2];
    auto b_load_dense = [&](int set, int t, int i0 = 0, int i1 = 4) {
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            const int row = st_r + 64 * i;
            const bool ok = t < T && row < b_rows;
            const uint32_t off = ok ? ((uint32_t)row * (uint32_t)p.K + (uint32_t)(ks0 + t) * kBK + st_p * 8) * 2u : kOutOfRange;
            breg[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, 0);
        }
    };
    auto b_load_packed = [&](int set, int c) {               // chunk c of this workgroup
        const bool in = 2 * c < T;
        const uint32_t kc = (uint32_t)(kc0 + c);
        // branch-free in wave-uniform values (a branch here would split the loop body and make its waits
        // conservative): group index by multiply-high plus a masked term, out of range by an added constant
        const uint32_t j = __umulhi(kc, p.cpg_inv) + (kc & p.cpg_one);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int nt = n0 / 16 + 2 * wave + q;
            const uint32_t skip = (in && nt * 16 < p.N) ? 0u : kOutOfRange;     // offsets stay below 2^31
            sreg[set][q] = __builtin_amdgcn_raw_buffer_load_b16(rs, ((uint32_t)(nt * 16 + nl) * (uint32_t)p.G + j) * 2u + skip, 0, 0);
#pragma unroll
            for (int kt = 0; kt < TPC; ++kt)
                breg[set][q * TPC + kt] = __builtin_amdgcn_raw_buffer_load_b128(
                    rb, ((uint32_t)nt * (uint32_t)p.KL + kc * TPC + kt) * 1024u + lane * 16 + skip, 0, 2 /* nt */);
        }
    };
    auto b_store_dense = [&](int set, int stage, int i0 = 0, int i1 = 4) {
#pragma unroll
        for (int i = i0; i < i1; ++i) *reinterpret_cast<u32x4_t*>(lds + stage * STAGE + A_BYTES + st_off + i * 8192) = breg[set][i];
    };
    // half = which 64 columns of the chunk; [q0, q1) x [o0, o1): tile-rows and 32-column operands to store
    auto b_store_packed = [&](int set, int half, int stage, int q0 = 0, int q1 = 2, int o0 = 0, int o1 = 2) {
#pragma unroll
        for (int q = q0; q < q1; ++q) {
            const half_t s = __builtin_bit_cast(half_t, sreg[set][q]);
            const half2_t s2 = {s, s};
            const int row = (2 * wave + q) * 16 + nl;
#pragma unroll
            for (int o = o0; o < o1; ++o) {                              // two 32-column MFMA operands per half
                Half8Words h;
                if constexpr (BSRC == 4) h.v = unpack_word4(breg[set][q][2 * half + o], magic);
                else h.v = unpack_words8(breg[set][q * 2 + half][2 * o], breg[set][q * 2 + half][2 * o + 1]);
#pragma unroll
                for (int e = 0; e < 4; ++e) h.h2[e] = h.h2[e] * s2;     // fp16(q * S)
                *reinterpret_cast<half8_t*>(lds + stage * STAGE + A_BYTES + swizzled(row, o * 4 + kq)) = h.v;
            }
        }
    };

    float4_t acc[MBW][4];
#pragma unroll
    for (int b = 0; b < MBW; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[b][r] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // operand rows of this lane: A rows wm*TM/2 + 16 b + nl, B rows wn*64 + 16 r + nl; (row & 7) == (nl & 7)
    const uint32_t a_rd = (uint32_t)((wm * (TM / 2) + nl) * 128);
    const uint32_t b_rd = (uint32_t)(A_BYTES + (wn * 64 + nl) * 128);
    half8_t bq[4];
    auto b_read = [&](int stage, int i) {                     // the wavefront's four weight operands of slice i
        const uint32_t po = (uint32_t)(((i * 4 + kq) ^ (nl & 7)) * 16);
#pragma unroll
        for (int r = 0; r < 4; ++r) bq[r] = *reinterpret_cast<const half8_t*>(lds + stage * STAGE + b_rd + r * 2048 + po);
    };
    auto compute_rows = [&](int stage, int i, int b0, int b1) {   // row blocks [b0, b1) of slice i against bq
        const uint32_t po = (uint32_t)(((i * 4 + kq) ^ (nl & 7)) * 16);
        half8_t a[MBW];
#pragma unroll
        for (int b = b0; b < b1; ++b) a[b] = *reinterpret_cast<const half8_t*>(lds + stage * STAGE + a_rd + b * 2048 + po);
#pragma unroll
        for (int b = b0; b < b1; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[b][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[b], bq[r], acc[b][r], 0, 0, 0);
    };

    // One step: arithmetic on stage (t & 1) while the next step's tiles go from registers into the other stage
    // and the loads of step t+1+PD (chunk c+PD) are issued.  u = t & 3 is a literal at every call site.
    auto step = [&](int u, int t) {
        const int stage = u & 1;
        const int set = PD == 2 ? (u & 1) : 0;               // register set that holds step t+1
        if constexpr (MBW == 8) {
            // tall tile: the step runs in four quarters (a 32-column slice x four of the eight row blocks), each with
            // 16 MFMAs that carry a quarter of the step's LDS stores, dequantisation and global loads between them;
            // at most four activation operands are live at a time (256 registers without spilling)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int i = qd >> 1, bh = qd & 1;
                if (bh == 0) b_read(stage, i);
                compute_rows(stage, i, bh * 4, bh * 4 + 4);
                a_store(set, stage ^ 1, qd, qd + 1);
                if constexpr (BSRC == 0) b_store_dense(set, stage ^ 1, qd, qd + 1);
                else b_store_packed(0, (u + 1) & 1, stage ^ 1, i, i + 1, bh, bh + 1);
                a_load(set, t + 1 + PD, qd, qd + 1);
                if constexpr (BSRC == 0) b_load_dense(set, t + 1 + PD, qd, qd + 1);
                else if (qd == 3 && (u & 1) == 0) b_load_packed(0, (t >> 1) + PD);
                if (bh == 0) __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                if constexpr (BSRC != 0) __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            return;
        }
        if constexpr (BSRC != 0 && MBW == 4) {
            // short packed tile: two halves (a 32-column slice each), each with 16 MFMAs that carry one tile-row to
            // dequantise, half of the activation staging and, every other step, the next chunk's loads
            const int cset = PD == 2 ? (((u + 1) >> 1) & 1) : 0;    // set of chunk (t+1) >> 1, stored half (t+1) & 1
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                b_read(stage, h);
                compute_rows(stage, h, 0, MBW);
                a_store(set, stage ^ 1, h, h + 1);
                b_store_packed(cset, (u + 1) & 1, stage ^ 1, h, h + 1);
                a_load(set, t + 1 + PD, h, h + 1);
                if (h == 1 && (u & 1) == 0) b_load_packed(cset, (t >> 1) + PD);   // the chunk just finished leaves its registers
                __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
                for (int o = 0; o < 2; ++o) {                            // one operand: 2 MFMAs per 4 vector ops, then its store
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                    if (o == 0) {
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            return;
        }
        // short dense tile: two halves, each with 16 MFMAs that carry three of the step's six LDS stores and global loads
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            b_read(stage, h);
            compute_rows(stage, h, 0, MBW);
            a_store(set, stage ^ 1, h, h + 1);
            b_store_dense(set, stage ^ 1, 2 * h, 2 * h + 2);
            a_load(set, t + 1 + PD, h, h + 1);
            b_load_dense(set, t + 1 + PD, 2 * h, 2 * h + 2);
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };

    // ---- prologue: step 0 into stage 0; registers then hold the next PD steps / chunks, issued in the loop's
    // order so that its waits are exact counts ----
    a_load(0, 0);
    if constexpr (BSRC == 0) b_load_dense(0, 0); else b_load_packed(0, 0);
    a_store(0, 0);
    if constexpr (BSRC == 0) b_store_dense(0, 0); else b_store_packed(0, 0, 0);
    if constexpr (BSRC == 0 && MBW == 8) {                   // the tall dense step issues its loads piece by piece
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            a_load(0, 1, qd, qd + 1);
            b_load_dense(0, 1, qd, qd + 1);
        }
    } else if constexpr (BSRC == 0) {                        // the short dense step issues its loads half by half
#pragma unroll
        for (int s = 0; s < PD; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a_load(s, 1 + s, h, h + 1);
                b_load_dense(s, 1 + s, 2 * h, 2 * h + 2);
            }
    } else {
        a_load(0, 1);
        if constexpr (PD == 2) {
            b_load_packed(1, 1);
            a_load(1, 2);
        }
    }
    __syncthreads();

    int t = 0;
    for (; t + 4 <= T; t += 4) {          // no control flow between steps: every wait inside is an exact count
        step(0, t);
        step(1, t + 1);
        step(2, t + 2);
        step(3, t + 3);
    }
    if (t < T) {                          // T is even
        step(0, t);
        step(1, t + 1);
    }

    // ---- store: lane holds rows 16 b + 4 kq + e, column 16 r + nl of its wavefront tile ----
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int n = n0 + wn * 64 + r * 16 + nl;
        if (n >= p.N) continue;
#pragma unroll
        for (int b = 0; b < MBW; ++b) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = m0 + wm * (TM / 2) + b * 16 + kq * 4 + e;
                if (m < p.M) {
                    if (p.split_k == 1) p.C[(int64_t)m * p.N + n] = (half_t)acc[b][r][e];
                    else p.ws[((int64_t)sg * p.M + m) * p.N + n] = acc[b][r][e];
                }
            }
        }
    }
}

template <int BSRC, int MBW>
hipError_t launch_tile_inst(const TileParams& tp, dim3 grid, hipStream_t st) {
    constexpr size_t lds = 2 * (size_t)(32 * MBW + kTN) * 128;
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tile_gemm_kernel<BSRC, MBW>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_done = true;
    }
    hipLaunchKernelGGL((tile_gemm_kernel<BSRC, MBW>), grid, dim3(kThreads), lds, st, tp);
    return hipGetLastError();
}

// rows16: 16-row blocks per wavefront (4 or 8), 0 = choose.
hipError_t launch_tile(TileParams& tp, int bsrc, int64_t M, int rows16, hipStream_t st) {
    // 128- or 256-row tiles: one workgroup runs per compute unit, so the launch takes rounds of 256 tiles; a 256-row
    // tile takes about 1.5 times as long as a 128-row one with packed weights (it halves the unpacking per flop) and
    // 1.7 times with dense ones, so it pays unless it wastes most of a round (measured on the 8B and 70B shapes at
    // 512 to 8192 rows).
    const int64_t xb = (tp.N + kTN - 1) / kTN;
    const int64_t r_short = (xb * ((M + 127) / 128) * tp.split_k + 255) / 256;
    const int64_t r_tall = (xb * ((M + 255) / 256) * tp.split_k + 255) / 256;
    const bool tall = rows16 ? rows16 == 8 : (M > 128 && (bsrc == 0 ? 1.7 : 1.5) * (double)r_tall < (double)r_short);
    const int tm = tall ? 256 : 128;
    tp.XB = (int)xb;
    tp.ZB = (int)((M + tm - 1) / tm);
    const int xb_pad = (tp.XB + kXcds - 1) / kXcds * kXcds;
    dim3 grid((unsigned)(xb_pad * tp.ZB), (unsigned)tp.split_k, 1);
    if (bsrc == 0) return tall ? launch_tile_inst<0, 8>(tp, grid, st) : launch_tile_inst<0, 4>(tp, grid, st);
    if (bsrc == 4) return tall ? launch_tile_inst<4, 8>(tp, grid, st) : launch_tile_inst<4, 4>(tp, grid, st);
    return tall ? launch_tile_inst<8, 8>(tp, grid, st) : launch_tile_inst<8, 4>(tp, grid, st);
}

void fill_common(TileParams& tp, const void* A, void* C, float* ws, int64_t M, int64_t N, int64_t K, int split_k) {
    tp.A = static_cast<const half_t*>(A);
    tp.C = static_cast<half_t*>(C);
    tp.ws = ws;
    tp.M = (int)M; tp.N = (int)N; tp.K = (int)K;
    tp.split_k = split_k;
    const int KC = (int)(K / kChunkK);
    tp.kc_base = KC / split_k;
    tp.kc_rem = KC % split_k;
}

}  // namespace

bool tile_plan_valid(const LinearArgs& a, const LinearPlan& p) {
    if (a.g % kChunkK != 0 || a.K % kChunkK != 0) return false;
    return p.split_k >= 1 && p.split_k <= a.K / kChunkK;
}

hipError_t launch_linear_tile(const LinearArgs& a, const LinearPlan& p, hipStream_t st) {
    TileParams tp;
    fill_common(tp, a.A, a.C, a.workspace, a.M, a.N, a.K, p.split_k);
    tp.B = a.qweight;
    tp.scales = static_cast<const half_t*>(a.scales);
    tp.G = (int)(a.K / a.g);
    tp.cpg = (int)(a.g / kChunkK);
    tp.cpg_inv = tp.cpg == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint32_t)tp.cpg) + 1u;
    tp.cpg_one = tp.cpg == 1 ? 0xFFFFFFFFu : 0u;
    tp.KL = (int)(a.K / (a.bits == 4 ? 128 : 64));
    tp.b_bytes = (uint32_t)((size_t)a.N * a.K * a.bits / 8);
    tp.sc_bytes = (uint32_t)((size_t)a.N * tp.G * 2);
    hipError_t e = launch_tile(tp, a.bits, a.M, p.m_rows16 == 4 || p.m_rows16 == 8 ? p.m_rows16 : 0, st);
    if (e != hipSuccess) return e;
    if (p.split_k > 1) e = launch_splitk_reduce(a.workspace, a.C, a.M * a.N, p.split_k, st);
    return e;
}

hipError_t launch_gemm_fp16(const void* A, const void* W, void* C, float* workspace, int64_t M, int64_t N, int64_t K,
                            int split_k, hipStream_t st) {
    TileParams tp;
    fill_common(tp, A, C, workspace, M, N, K, split_k);
    tp.B = W;
    tp.scales = static_cast<const half_t*>(W);           // unused by the dense source; any valid pointer
    tp.G = 1; tp.cpg = 1; tp.cpg_inv = 0; tp.cpg_one = 0xFFFFFFFFu; tp.KL = 0;
    tp.b_bytes = 0;
    tp.sc_bytes = 16;
    hipError_t e = launch_tile(tp, 0, M, 0, st);
    if (e != hipSuccess) return e;
    if (split_k > 1) e = launch_splitk_reduce(workspace, C, M * N, split_k, st);
    return e;
}

}  // namespace rtn
