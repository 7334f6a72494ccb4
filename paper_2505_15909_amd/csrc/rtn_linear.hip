// Fused dequantise-GEMM of the RTN weight-only quantised linear layer for gfx950
// (Sections 2.3 and 5: 16-bit activations times 4-/8-bit weights at token-generation batch
// sizes, where every weight byte is used once and time = weight bytes / HBM bandwidth).
//
//   C[m, n] = fp16( sum_k A[m, k] * q[n, k] * S[n, k / g] )
//
// Skinny MFMA kernel.  A workgroup is WN x WK wavefronts: wavefront (wn, wk) owns one tile-row
// (16 output channels) and a contiguous run of k-chunks (4 tiles = 4 KiB of packed codes each)
// of the workgroup's K range.  Per chunk it issues four 16-byte-per-lane loads (1 KiB per
// wavefront each, fully coalesced), unpacks the codes in registers to exact fp16 integers and
// feeds them as the B operand of v_mfma_f32_16x16x32_f16.  The A operand is the activation
// block staged per workgroup in LDS (padded rows) and read 16 bytes per lane right before each
// MFMA; lanes of batch rows beyond M read the last valid row (output rows never mix in a matrix
// product, and those rows are not stored).  The slice goes from global memory straight into LDS
// (buffer_load ... lds: no registers, no LDS store instructions, every address wave-uniform
// arithmetic) and is requested before the first weight load; a workgroup one wavefront wide along
// N stages per wavefront and needs no barrier before the main loop.  A slice that does not fit one
// stage alternates between two LDS buffers, the next stage's loads in flight while the current one
// is consumed, one barrier per stage.
// Scales multiply the fp32 partial sum of each group (exact codes into the matrix cores, one
// fp32 multiply-add per group and output), never the individual weights.  The WK partial
// results of a tile-row are summed through LDS in a fixed order; an optional global split-K
// writes fp32 partials to the workspace and a second kernel sums them in a fixed order, so
// results are bit-reproducible.
//
// Memory pipeline.  All global reads go through buffer resources: a load whose offset is
// beyond the resource's size returns zero without touching memory, so loads that fall outside
// a wavefront's share (tail chunks, padding rows, padding tile-rows) are issued anyway with an
// out-of-range offset.  Every wavefront therefore issues the same loads in the same order on
// every path, which lets the compiler wait with exact vmcnt values instead of draining the
// queue, and NB register buffers rotate so that NB-1 chunks are in flight while one is
// consumed.  The activation loads are issued before the weight loads so that staging does
// not wait behind the (longer) HBM latency of the weights: loads complete in order, so waiting
// until only the weight loads issued after them are outstanding means the staged rows have landed.
//
// MFMA operand maps (16x16x32 f16): a-operand lane l = row l % 16, k-slot l / 16 (8 halves);
// b-operand lane l = column l % 16, same k-slot; result lane l, register e = row 4 (l/16) + e,
// column l % 16.  Rows are batch entries m, columns are output channels n, so every lane needs
// exactly one scale per group (that of its own weight row).
#include "rtn_device.h"
#include "rtn_internal.h"
#include <vector>

namespace rtn {

constexpr int kChunkTiles = 4;            // tiles (16-byte loads per lane) per k-chunk
constexpr int kLdsPadHalves = 8;          // row stride = 16 bytes mod 256 bytes: conflict-free b128 reads
constexpr uint32_t kOutOfRange = 0x7FFF0000u;   // beyond any resource size used here (< 2 GiB)
constexpr int kBufferFlags = 0x00020000;  // raw buffer, 32-bit data format

struct SkinnyParams {
    const half_t* A;
    const uint8_t* qw;
    const half_t* scales;
    const half_t* zeros;   // asymmetric variant only (ZP)
    half_t* C;
    float* ws;
    int M, N, K;
    int G;            // groups per row
    int g;            // group size
    int NT;           // N / 16
    int KL;           // tiles per row
    int KC;           // chunks per row
    int WN, WK;            // wave = wk * WN + wn; any WN x WK <= 16
    uint32_t wn_inv;       // floor(2^32 / WN) + 1: wave -> wk by multiply-high (unused when WN == 1)
    int split_k;
    int kc_base, kc_rem;   // workgroup sg covers chunks [sg*kc_base + min(sg, kc_rem), ...): KC split evenly
    uint32_t cpg_inv;      // floor(2^32 / (g / CK)) + 1 when g > CK (0 when g == CK): chunk -> group by multiply-high
    int per;          // chunks per wavefront (largest)
    int nstage;       // activation stages (1 unless MULTI)
    int sc;           // chunks per wavefront per stage (single stage: the wavefront's whole share)
    uint32_t sc_inv, rpr_inv;   // floor(2^32 / sc) + 1, floor(2^32 / (WK sc)) + 1: exact division of small indices (unused when the divisor is 1)
    int stage_row_step;         // wavefronts that share one column run of the staged rows (fewer runs per row than wavefronts)
    int stage_halves; // halves between the two LDS buffers of the staged mode
    int lds_stride;   // halves per staged activation row = WK * sc * CK + pad
    uint32_t qw_bytes, sc_bytes, a_bytes;
};

template <int BITS>
struct Geom {
    static constexpr int TK = Layout<BITS>::TK;
    static constexpr int MPT = Layout<BITS>::MFMA_PER_TILE;
    static constexpr int CK = kChunkTiles * TK;           // k per chunk: 512 / 256
    static constexpr int NM = kChunkTiles * MPT;          // MFMAs per chunk: 16 / 8
};

// The fp16 scales of one k-chunk of one weight row: NGC = groups per chunk = 1, 2, 4, 8 or 16 consecutive values.
struct ScaleOct { u32x4_t v[2]; };
template <int NGC> struct ScaleVec;
template <> struct ScaleVec<1> { typedef uint16_t raw_t; };
template <> struct ScaleVec<2> { typedef uint32_t raw_t; };
template <> struct ScaleVec<4> { typedef u32x2_t raw_t; };
template <> struct ScaleVec<8> { typedef u32x4_t raw_t; };
template <> struct ScaleVec<16> { typedef ScaleOct raw_t; };

template <int NGC>
__device__ __forceinline__ float scale_at(const typename ScaleVec<NGC>::raw_t& raw, int i) {
    if constexpr (NGC == 1) {
        return (float)__builtin_bit_cast(half_t, raw);
    } else if constexpr (NGC == 2) {
        half2_t h = __builtin_bit_cast(half2_t, raw);
        return (float)h[i];
    } else {
        uint32_t word;                         // by value: bit_cast of a vector-element lvalue reads element 0
        if constexpr (NGC == 16) word = raw.v[i >> 3][(i >> 1) & 3];
        else word = raw[i >> 1];
        half2_t h = __builtin_bit_cast(half2_t, word);
        return (float)h[i & 1];
    }
}

template <int NGC>
__device__ __forceinline__ typename ScaleVec<NGC>::raw_t load_scales(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    if constexpr (NGC == 1) return __builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
    else if constexpr (NGC == 2) return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
    else if constexpr (NGC == 4) return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
    else if constexpr (NGC == 8) return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    else {
        ScaleOct o;                            // out-of-range offsets stay out of range: the resource is < 2 GiB
        o.v[0] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        o.v[1] = __builtin_amdgcn_raw_buffer_load_b128(r, off + 16, 0, 0);
        return o;
    }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// MULTI = false: the workgroup's whole activation slice is staged once, before the main loop.
// MULTI = true: it is staged sc chunks per wavefront at a time, one stage ahead, in two alternating LDS buffers.
// MB: 16-row activation blocks per wavefront (batch rows per workgroup = 16 MB); every unpacked weight
// operand feeds MB MFMAs, so the weights are streamed once for up to 16 MB batch rows.
// DOT = true (M <= 4, MB = 1): the same wavefront layout, but the products are done by the vector ALU
// (v_dot2_f32_f16, 4 per weight word and batch row; lane l accumulates row l % 16 over its own k-slots
// and the four k-slot lanes of a row are summed by two cross-lane adds at the end) instead of the matrix
// cores -- the wavefront-reduction GEMV the skinny MFMA path is measured against.
// The body takes the workgroup's coordinates as arguments so that one launch can also serve several independent
// problems (grouped launch below).
template <int BITS, int NGC, int NB, bool MULTI, int MB, bool DOT, bool ZP = false>
__device__ __forceinline__ void skinny_body(const SkinnyParams& p, const int bx, const int by, const int bz) {
    typedef Geom<BITS> GM;
    typedef typename ScaleVec<NGC>::raw_t sraw_t;
    extern __shared__ __align__(16) uint8_t lds_bytes[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept scalar
    const int wk = p.WN == 1 ? wave : (int)__umulhi((uint32_t)wave, p.wn_inv), wn = wave - wk * p.WN;   // scalar
    const int nl = lane & 15, kq = lane >> 4;

    constexpr int MROWS = 16 * MB;                                      // batch rows per workgroup
    const int m0 = bz * MROWS;
    const int Mb = min(MROWS, p.M - m0);
    const int sg = by;
    const int cb0 = sg * p.kc_base + min(sg, p.kc_rem);               // chunk range of this workgroup
    const int cb1 = cb0 + p.kc_base + (sg < p.kc_rem ? 1 : 0);
    const int cw0 = min(cb0 + wk * p.per, cb1), cw1 = min(cw0 + p.per, cb1);   // ... and of this wavefront
    const int nt = bx * p.WN + wn;
    const bool nt_ok = nt < p.NT;

    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.qw), 0, p.qw_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p.scales), 0, p.sc_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(p.A), 0, p.a_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(ZP ? p.zeros : p.scales), 0, p.sc_bytes, kBufferFlags);
    const uint32_t w_lane = (uint32_t)nt * (uint32_t)p.KL * 1024u + lane * 16;
    const uint32_t s_lane = ((uint32_t)nt * 16 + nl) * (uint32_t)p.G * 2u;
    const uint32_t magic = fp16_magic_vgpr();

    // ---- activation staging --------------------------------------------------------------------
    // A stage holds, for every row and every K-wavefront w, the sc chunks that wavefront w consumes in this stage:
    // LDS [row][w][sc * CK] (+ pad).  It goes from global memory straight into LDS (buffer_load ... lds, 16 bytes per
    // lane, no registers): one instruction moves a run = one k-chunk of one staged row (64 lanes x 16 bytes at 4 bit, 32
    // lanes at 8 bit).  Runs are dealt to the wavefronts by (column run, row) so that every address is wave-uniform
    // arithmetic.  Runs past a wavefront's share are skipped (nothing reads them).
    //   Single stage (MULTI = false): the compiler's builtin, issued before everything else.
    //   Staged (MULTI = true): two LDS buffers; the loads of stage s + 1 are issued while stage s is consumed.  The
    //   compiler must not see them -- it would make every later LDS read wait for them, since it cannot tell the two
    //   buffers apart -- so they go out as inline assembly (M0 = LDS address of the run, saved and restored) and the
    //   waits are explicit: loads complete in order, so once at most the NB chunks requested after them are outstanding
    //   they have landed.
    half_t* lds_a = reinterpret_cast<half_t*>(lds_bytes);
    constexpr int RP = GM::CK / 8;                                   // lanes (16-byte pieces) per run
    const int nwaves = p.WN * p.WK;                                   // (not blockDim: that is one more scalar load and wait)
    const int rpr = p.WK * p.sc;                                      // runs per staged row
    int col0, col_step, row0, row_step, col_end = rpr;
    if (p.WN == 1) {
        // every wavefront has a K-slice of its own: it stages just that (no other wavefront reads it, no barrier)
        col0 = wk * p.sc; col_step = 1; col_end = col0 + p.sc; row0 = 0; row_step = 1;
    } else if (rpr >= nwaves) {
        col0 = wave; col_step = nwaves; row0 = 0; row_step = 1;
    } else {
        // fewer runs per row than wavefronts: stage_row_step = nwaves / rpr wavefronts take the rows of one column run in turn
        row0 = rpr == 1 ? wave : (int)__umulhi((uint32_t)wave, p.rpr_inv); row_step = p.stage_row_step;
        col0 = wave - row0 * rpr; col_step = rpr;
        if (row0 >= row_step) col_end = 0;                            // left-over wavefronts stage nothing
    }
    const uint32_t lane_off = lane * 16;
    auto stage_issue = [&](int s, uint32_t buf_bytes) {
        if (RP == 64 || lane < RP) {
            for (int col = col0; col < col_end; col += col_step) {
                const int w = p.sc == 1 ? col : (int)__umulhi((uint32_t)col, p.sc_inv), j = col - w * p.sc;
                const int c0 = min(cb0 + w * p.per, cb1), c1 = min(c0 + p.per, cb1);
                const int c = c0 + s * p.sc + j;
                if (c < c1) {
                    for (int row = row0; row < Mb; row += row_step) {
                        const uint32_t soff = ((uint32_t)(m0 + row) * (uint32_t)p.K + (uint32_t)c * GM::CK) * 2u;
                        const uint32_t ldsoff = buf_bytes + (uint32_t)(row * p.lds_stride + col * GM::CK) * 2u;
                        if constexpr (MULTI) {
                            uint32_t keep_m0;
                            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                                         "buffer_load_dwordx4 %2, %3, %4 offen lds\n\ts_nop 0\n\ts_mov_b32 m0, %0"
                                         : "=&s"(keep_m0) : "s"(ldsoff), "v"(lane_off), "s"(ra), "s"(soff) : "memory");
                        } else {
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void*)(lds_bytes + ldsoff), 16,
                                                                     lane_off, soff, 0, 0);
                        }
                    }
                }
            }
        }
    };

    // ---- weight / scale prefetch: NB chunks in flight --------------------------------------------
    u32x4_t wbuf[NB][kChunkTiles];
    sraw_t sbuf[NB];
    sraw_t zbuf[ZP ? NB : 1];             // zero points, same shape and offsets as the scales
    (void)zbuf;
    (void)rz;
    auto fetch = [&](int j, int ci) {
        const bool ok = nt_ok && ci < cw1;                            // wave-uniform
        const uint32_t si = (NGC > 1) ? (uint32_t)ci * NGC : (p.cpg_inv == 0 ? (uint32_t)ci : __umulhi((uint32_t)ci, p.cpg_inv));
        const uint32_t so = ok ? s_lane + si * 2u : kOutOfRange;
        const uint32_t wo = ok ? w_lane + (uint32_t)ci * (kChunkTiles * 1024u) : kOutOfRange;
        sbuf[j] = load_scales<NGC>(rs, so);                           // scales first: never the last to arrive
        if constexpr (ZP) zbuf[j] = load_scales<NGC>(rz, so);
#pragma unroll
        for (int c = 0; c < kChunkTiles; ++c)
            wbuf[j][c] = __builtin_amdgcn_raw_buffer_load_b128(rw, wo + c * 1024, 0, 2 /* nt: read-once stream */);
    };

    constexpr int LPC = ((NGC == 16) ? 2 : 1) * (ZP ? 2 : 1) + kChunkTiles;   // loads per fetch()
    stage_issue(0, 0u);                   // activation loads first: the oldest loads in flight
#pragma unroll
    for (int j = 0; j < NB; ++j) fetch(j, cw0 + j);
    wait_vmcnt<NB * LPC>();               // the staging loads are older than the NB chunks just requested
    if (p.WN > 1) __syncthreads();        // (one wavefront along N: every wavefront reads only what it staged itself)

    // ---- main loop -------------------------------------------------------------------------------
    float4_t acc[MB];
    const half_t* arow[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        acc[b] = (float4_t){0.f, 0.f, 0.f, 0.f};
        arow[b] = lds_a + min(b * 16 + nl, Mb - 1) * p.lds_stride + (wk * p.sc) * GM::CK + kq * 8;
    }
    const half_t* adot = lds_a + (wk * p.sc) * GM::CK + kq * 8;   // DOT: row 0 of this k-slot
    (void)adot;
    int ci = cw0;
    for (int s = 0; s < p.nstage; ++s) {
        int aoff = MULTI ? (s & 1) * p.stage_halves : 0;              // which LDS buffer this stage reads
        bool next_issued = !MULTI || s + 1 >= p.nstage;
        for (int u = 0; u < p.sc; u += NB) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                if (ci < cw1) {                                       // scalar branch, no loads inside
                    constexpr int MPG = GM::NM / NGC;                 // MFMAs (weight words per lane) per group
                    if constexpr (DOT) {
#pragma unroll
                        for (int gi = 0; gi < NGC; ++gi) {
                            float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int q = 0; q < MPG; ++q) {
                                const int i = gi * MPG + q;
                                Half8Words bw;
                                bw.v = unpack_operand<BITS>(wbuf[j][i / GM::MPT], i % GM::MPT, magic);
#pragma unroll
                                for (int m = 0; m < 4; ++m) {
                                    if (m < Mb) {                     // uniform
                                        Half8Words a;                 // same address for the 16 lanes of a k-slot
                                        a.v = *reinterpret_cast<const half8_t*>(adot + m * p.lds_stride + aoff + i * 32);
#pragma unroll
                                        for (int h = 0; h < 4; ++h)
                                            part[m] = __builtin_amdgcn_fdot2(a.h2[h], bw.h2[h], part[m], false);
                                    }
                                }
                            }
                            const float sc = scale_at<NGC>(sbuf[j], gi);
#pragma unroll
                            for (int m = 0; m < 4; ++m) acc[0][m] = fmaf(sc, part[m], acc[0][m]);
                        }
                    } else {
#pragma unroll
                        for (int gi = 0; gi < NGC; ++gi) {
                            float4_t part[MB];
#pragma unroll
                            for (int b = 0; b < MB; ++b) part[b] = (float4_t){0.f, 0.f, 0.f, 0.f};
                            float zp = 0.0f;
                            if constexpr (ZP) zp = scale_at<NGC>(zbuf[j], gi);
                            (void)zp;
#pragma unroll
                            for (int q = 0; q < MPG; ++q) {
                                const int i = gi * MPG + q;
                                half8_t bw;
                                if constexpr (ZP) bw = unpack_operand_zp<BITS>(wbuf[j][i / GM::MPT], i % GM::MPT, magic, zp);
                                else bw = unpack_operand<BITS>(wbuf[j][i / GM::MPT], i % GM::MPT, magic);
#pragma unroll
                                for (int b = 0; b < MB; ++b) {
                                    const half8_t a = *reinterpret_cast<const half8_t*>(arow[b] + aoff + i * 32);
                                    part[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bw, part[b], 0, 0, 0);
                                }
                            }
                            const float sc = scale_at<NGC>(sbuf[j], gi);
#pragma unroll
                            for (int b = 0; b < MB; ++b)
#pragma unroll
                                for (int e = 0; e < 4; ++e) acc[b][e] = fmaf(sc, part[b][e], acc[b][e]);
                        }
                    }
                }
                if constexpr (MULTI) {
                    // the next stage's activations, into the other buffer: issued after the stage's first chunk is consumed
                    // (with one chunk in flight nothing is outstanding at this point, so no later wait sees these loads)
                    if (!next_issued) {
                        stage_issue(s + 1, (uint32_t)(((s + 1) & 1) * p.stage_halves) * 2u);
                        next_issued = true;
                    }
                }
                fetch(j, ci + NB);        // unconditional: out of range past the wavefront's share
                aoff += GM::CK;
                ++ci;
            }
        }
        if constexpr (MULTI) {
            if (s + 1 < p.nstage) {       // uniform: the next stage has landed, and everyone is done reading this one
                wait_vmcnt<NB * LPC>();
                if (p.WN > 1) __syncthreads();
            }
        }
    }

    if constexpr (DOT) {                  // sum the four k-slot lanes of every weight row (fixed order)
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float v = acc[0][m];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[0][m] = v;
        }
    }

    // ---- in-workgroup split-K reduction (fixed order) ------------------------------------------
    if (p.WK > 1) {
        __syncthreads();                  // everyone is done reading the staged activations
        float4_t* red = reinterpret_cast<float4_t*>(lds_bytes);
        if (wk > 0) {
#pragma unroll
            for (int b = 0; b < MB; ++b) red[(((wk - 1) * p.WN + wn) * MB + b) * 64 + lane] = acc[b];
        }
        __syncthreads();
        if (wk == 0) {
            for (int w = 1; w < p.WK; ++w) {
#pragma unroll
                for (int b = 0; b < MB; ++b) {
                    const float4_t v = red[(((w - 1) * p.WN + wn) * MB + b) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[b][e] += v[e];
                }
            }
        }
    }
    if (wk != 0 || !nt_ok) return;

    // ---- store: lane holds rows m = 16 b + 4 kq + e (DOT: rows m = e, in the lanes of k-slot 0), column
    // n = 16 tile + nl --------------------------------------------------------------------------------
    const int n = nt * 16 + nl;
#pragma unroll
    for (int b = 0; b < MB; ++b) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = DOT ? e : b * 16 + kq * 4 + e;
            if (m < Mb && (!DOT || kq == 0)) {
                if (p.split_k == 1) p.C[(int64_t)(m0 + m) * p.N + n] = (half_t)acc[b][e];
                else p.ws[((int64_t)sg * p.M + (m0 + m)) * p.N + n] = acc[b][e];
            }
        }
    }
}

template <int BITS, int NGC, int NB, bool MULTI, int MB, bool DOT = false, bool ZP = false>
__global__ __launch_bounds__(1024) void skinny_mfma_kernel(const SkinnyParams p) {
    // Every argument the prologue needs is requested here, together, behind one wait: left alone the compiler loads
    // them where they are first used, four scalar-cache round trips in a row before the first memory request goes out
    // (measured: 1 % of the Llama-8B layer set).
    asm volatile("" :: "s"(p.A), "s"(p.qw), "s"(p.scales), "s"(p.M), "s"(p.K), "s"(p.G), "s"(p.NT), "s"(p.KL), "s"(p.WN), "s"(p.WK), "s"(p.wn_inv),
                 "s"(p.kc_base), "s"(p.kc_rem), "s"(p.cpg_inv), "s"(p.per), "s"(p.sc), "s"(p.sc_inv), "s"(p.rpr_inv), "s"(p.stage_row_step),
                 "s"(p.lds_stride), "s"(p.qw_bytes), "s"(p.sc_bytes), "s"(p.a_bytes));
    skinny_body<BITS, NGC, NB, MULTI, MB, DOT, ZP>(p, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Grouped launch: up to kMaxGroup independent problems of the same precision, group size and workgroup shape
// and activation staging mode (e.g. the experts of a mixture-of-experts layer, or modules that do not feed one another) in one grid.
// Workgroup b belongs to the problem g with first_block[g] <= b < first_block[g + 1].
constexpr int kMaxGroup = 16;
struct GroupedParams {
    int n;
    int first_block[kMaxGroup + 1];
    SkinnyParams p[kMaxGroup];
};

template <int BITS, int NGC, bool MULTI>
__global__ __launch_bounds__(1024) void skinny_grouped_kernel(const GroupedParams gp) {
    const int b = blockIdx.x;
    int g = 0;
    for (int i = 1; i < gp.n; ++i) g = (b >= gp.first_block[i]) ? i : g;     // uniform
    skinny_body<BITS, NGC, 1, MULTI, 1, false>(gp.p[g], b - gp.first_block[g], 0, 0);
}

// Sums the split-K partials in a fixed order (s = 0, 1, 2, ...) and rounds once to fp16.  The partials of a batch of up
// to eight splits are requested together and summed as they arrive: a loop of load-wait-add takes one memory round trip
// per split (4 us for four splits of a 16 x 4096 output, against 1.5 us for the whole kernel this way).
// S > 0: exactly S splits (S <= 8), fully unrolled.  S = 0: any number, in batches of eight.
template <int S>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ ws, half_t* __restrict__ C,
                                                            int64_t MN, int split_k) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= MN) return;                                  // MN is a multiple of 16
    const float* src = ws + i;
    float4_t v;
    if constexpr (S > 0) {
        float4_t part[S];
#pragma unroll
        for (int s = 0; s < S; ++s) part[s] = *reinterpret_cast<const float4_t*>(src + (int64_t)s * MN);
        v = part[0];
#pragma unroll
        for (int s = 1; s < S; ++s) v += part[s];
    } else {
        v = (float4_t){0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < split_k; s0 += 8) {         // uniform
            float4_t part[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)                   // past the last split: partial 0 again (a valid address), not added
                part[u] = *reinterpret_cast<const float4_t*>(src + (int64_t)(s0 + u < split_k ? s0 + u : 0) * MN);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (s0 + u == 0) v = part[0];             // the first term starts the sum (no 0 + x: keeps the sign of zero)
                else if (s0 + u < split_k) v += part[u];
            }
        }
    }
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    half4_t h = {(half_t)v[0], (half_t)v[1], (half_t)v[2], (half_t)v[3]};
    *reinterpret_cast<half4_t*>(C + i) = h;
}

// Geometry the kernel and the LDS budget share: chunks per wavefront, chunks per wavefront per
// activation stage, number of stages.  A slice that fits kSingleStageLds is staged at once (a
// wavefront's exact share); otherwise it is staged a power of two of chunks at a time (at least the
// prefetch depth) in two alternating LDS buffers of at most kMultiStageLds each (so that two
// workgroups still share a compute unit).
constexpr size_t kSingleStageLds = 150 * 1024;         // direct-to-LDS staging needs no registers: one stage may take (almost) the whole LDS
constexpr size_t kMultiStageLds = 32 * 1024 + 1024;
constexpr size_t kMultiStageLdsWide = 72 * 1024;       // more than 16 activation rows: one chunk of 64 rows

struct StageGeom {
    int per, sc, nstage, rows;
    bool multi, fits;
    size_t lds, stage_bytes;
};

static StageGeom stage_geometry(const LinearArgs& a, const LinearPlan& p) {
    const int ck = (a.bits == 4) ? 512 : 256;
    const int kc = (int)(a.K / ck);
    const int blk = (kc + p.split_k - 1) / p.split_k;                 // chunks per workgroup
    StageGeom g;
    g.per = (blk + p.waves_k - 1) / p.waves_k;
    const int mrows = 16 * p.m_rows16;                               // batch rows per workgroup
    g.rows = (int)(a.M < mrows ? a.M : mrows);
    const size_t red = p.waves_k > 1 ? (size_t)(p.waves_k - 1) * p.waves_n * p.m_rows16 * 1024 : 0;
    auto bytes_of = [&](int sc) { return ((size_t)g.rows * ((size_t)p.waves_k * sc * ck + kLdsPadHalves) * 2 + 15) & ~(size_t)15; };
    const int sc_full = g.per;                                        // whole share in one stage
    int sc = sc_full;
    g.fits = true;
    g.multi = false;
    if (bytes_of(sc_full) > kSingleStageLds) {
        // largest stage within the budget; failing that, the smallest one if two of it still fit the LDS
        int m = 1;
        while (m * 2 < sc_full) m *= 2;                               // stages of a power of two of chunks
        const size_t budget = g.rows > 16 ? kMultiStageLdsWide : kMultiStageLds;
        while (m > p.prefetch && bytes_of(m) > budget) m /= 2;
        if (m >= p.prefetch && m > 0 && 2 * bytes_of(m) <= kMaxLdsBytes) {
            g.multi = true;
            sc = m;
        } else {
            g.fits = bytes_of(sc_full) <= kMaxLdsBytes;               // one large stage
        }
    }
    g.sc = sc;
    g.nstage = g.multi ? (g.per + sc - 1) / sc : 1;
    g.stage_bytes = bytes_of(sc);
    const size_t bytes = g.multi ? 2 * g.stage_bytes : g.stage_bytes;
    g.lds = bytes > red ? bytes : red;
    return g;
}

bool linear_plan_fits(const LinearArgs& a, const LinearPlan& p, size_t lds_limit) {
    const StageGeom g = stage_geometry(a, p);
    if (p.path == 2 && g.multi) return false;            // the dot-product variant stages once
    return g.fits && g.lds <= lds_limit;
}

size_t linear_lds_bytes(const LinearArgs& a, const LinearPlan& p) { return stage_geometry(a, p).lds; }

template <typename K>
static void allow_large_lds(K kernel) {
    static bool done = false;             // per instantiation
    if (!done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)kMaxLdsBytes);
        done = true;
    }
}

template <int BITS, int NGC, int NB, bool MULTI, int MB>
static void launch_skinny_inst(const SkinnyParams& sp, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    if constexpr (NGC <= Geom<BITS>::NM) {     // at most one group per MFMA (32 columns)
        allow_large_lds(skinny_mfma_kernel<BITS, NGC, NB, MULTI, MB>);
        hipLaunchKernelGGL((skinny_mfma_kernel<BITS, NGC, NB, MULTI, MB>), grid, block, lds, st, sp);
    }
}

template <int BITS, int NB, bool MULTI, int MB>
static hipError_t launch_skinny_ngc(const SkinnyParams& sp, int ngc, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    switch (ngc) {
        case 1: launch_skinny_inst<BITS, 1, NB, MULTI, MB>(sp, grid, block, lds, st); break;
        case 2: launch_skinny_inst<BITS, 2, NB, MULTI, MB>(sp, grid, block, lds, st); break;
        case 4: launch_skinny_inst<BITS, 4, NB, MULTI, MB>(sp, grid, block, lds, st); break;
        case 8: launch_skinny_inst<BITS, 8, NB, MULTI, MB>(sp, grid, block, lds, st); break;
        case 16: launch_skinny_inst<BITS, 16, NB, MULTI, MB>(sp, grid, block, lds, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_dot(const SkinnyParams& sp, int ngc, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    switch (ngc) {
        case 1:
            allow_large_lds(skinny_mfma_kernel<BITS, 1, 1, false, 1, true>);
            hipLaunchKernelGGL((skinny_mfma_kernel<BITS, 1, 1, false, 1, true>), grid, block, lds, st, sp);
            break;
        case 2:
            allow_large_lds(skinny_mfma_kernel<BITS, 2, 1, false, 1, true>);
            hipLaunchKernelGGL((skinny_mfma_kernel<BITS, 2, 1, false, 1, true>), grid, block, lds, st, sp);
            break;
        default:
            allow_large_lds(skinny_mfma_kernel<BITS, 4, 1, false, 1, true>);
            hipLaunchKernelGGL((skinny_mfma_kernel<BITS, 4, 1, false, 1, true>), grid, block, lds, st, sp);
            break;
    }
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_skinny(const SkinnyParams& sp, int ngc, int nb, bool multi, int mb, dim3 grid, dim3 block,
                                size_t lds, hipStream_t st) {
    if (mb == 4) return multi ? launch_skinny_ngc<BITS, 1, true, 4>(sp, ngc, grid, block, lds, st)
                              : launch_skinny_ngc<BITS, 1, false, 4>(sp, ngc, grid, block, lds, st);
    if (mb == 2) return multi ? launch_skinny_ngc<BITS, 1, true, 2>(sp, ngc, grid, block, lds, st)
                              : launch_skinny_ngc<BITS, 1, false, 2>(sp, ngc, grid, block, lds, st);
    if (nb == 1) return multi ? launch_skinny_ngc<BITS, 1, true, 1>(sp, ngc, grid, block, lds, st)
                              : launch_skinny_ngc<BITS, 1, false, 1>(sp, ngc, grid, block, lds, st);
    if (nb == 2) return multi ? launch_skinny_ngc<BITS, 2, true, 1>(sp, ngc, grid, block, lds, st)
                              : launch_skinny_ngc<BITS, 2, false, 1>(sp, ngc, grid, block, lds, st);
    return multi ? launch_skinny_ngc<BITS, 4, true, 1>(sp, ngc, grid, block, lds, st)
                 : launch_skinny_ngc<BITS, 4, false, 1>(sp, ngc, grid, block, lds, st);
}

// Asymmetric variant (per-group zero points): one chunk in flight, one 16-row block per wavefront.
template <int BITS, int NGC>
static void launch_skinny_zp_inst(const SkinnyParams& sp, bool multi, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    if constexpr (NGC <= Geom<BITS>::NM) {
        if (multi) {
            allow_large_lds(skinny_mfma_kernel<BITS, NGC, 1, true, 1, false, true>);
            hipLaunchKernelGGL((skinny_mfma_kernel<BITS, NGC, 1, true, 1, false, true>), grid, block, lds, st, sp);
        } else {
            allow_large_lds(skinny_mfma_kernel<BITS, NGC, 1, false, 1, false, true>);
            hipLaunchKernelGGL((skinny_mfma_kernel<BITS, NGC, 1, false, 1, false, true>), grid, block, lds, st, sp);
        }
    }
}

template <int BITS>
static hipError_t launch_skinny_zp(const SkinnyParams& sp, int ngc, bool multi, dim3 grid, dim3 block, size_t lds,
                                   hipStream_t st) {
    switch (ngc) {
        case 1: launch_skinny_zp_inst<BITS, 1>(sp, multi, grid, block, lds, st); break;
        case 2: launch_skinny_zp_inst<BITS, 2>(sp, multi, grid, block, lds, st); break;
        case 4: launch_skinny_zp_inst<BITS, 4>(sp, multi, grid, block, lds, st); break;
        case 8: launch_skinny_zp_inst<BITS, 8>(sp, multi, grid, block, lds, st); break;
        case 16: launch_skinny_zp_inst<BITS, 16>(sp, multi, grid, block, lds, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Everything a skinny-kernel launch needs, derived from the problem and its plan.
struct SkinnyLaunch {
    SkinnyParams sp;
    dim3 grid, block;
    size_t lds;
    int ngc;
    bool multi;
};

static SkinnyLaunch prepare_skinny(const LinearArgs& a, const LinearPlan& p) {
    const int tk = (a.bits == 4) ? 128 : 64;
    const int ck = kChunkTiles * tk;
    SkinnyLaunch L;
    SkinnyParams& sp = L.sp;
    sp.A = static_cast<const half_t*>(a.A);
    sp.qw = static_cast<const uint8_t*>(a.qweight);
    sp.scales = static_cast<const half_t*>(a.scales);
    sp.zeros = static_cast<const half_t*>(a.zeros);
    sp.C = static_cast<half_t*>(a.C);
    sp.ws = a.workspace;
    sp.M = (int)a.M; sp.N = (int)a.N; sp.K = (int)a.K;
    sp.g = (int)a.g;
    sp.G = (int)(a.K / a.g);
    sp.NT = (int)(a.N / 16);
    sp.KL = (int)(a.K / tk);
    sp.KC = (int)(a.K / ck);
    sp.WN = p.waves_n; sp.WK = p.waves_k;
    sp.wn_inv = p.waves_n == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint32_t)p.waves_n) + 1u;
    sp.split_k = p.split_k;
    sp.kc_base = sp.KC / p.split_k;
    sp.kc_rem = sp.KC % p.split_k;
    {
        const uint32_t cpg = (a.g >= ck) ? (uint32_t)(a.g / ck) : 1u;      // chunks per group
        sp.cpg_inv = cpg == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / cpg) + 1u;    // 0: one chunk per group
    }
    const StageGeom sgm = stage_geometry(a, p);
    sp.per = sgm.per;
    sp.sc = sgm.sc;
    sp.sc_inv = sgm.sc == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint32_t)sgm.sc) + 1u;
    sp.rpr_inv = p.waves_k * sgm.sc == 1 ? 0u : (uint32_t)(((uint64_t)1 << 32) / (uint32_t)(p.waves_k * sgm.sc)) + 1u;
    sp.stage_row_step = (p.waves_n * p.waves_k) / (p.waves_k * sgm.sc) > 0 ? (p.waves_n * p.waves_k) / (p.waves_k * sgm.sc) : 1;
    sp.nstage = sgm.nstage;
    sp.stage_halves = (int)(sgm.stage_bytes / 2);
    sp.lds_stride = p.waves_k * sgm.sc * ck + kLdsPadHalves;
    sp.qw_bytes = (uint32_t)((size_t)a.N * a.K * a.bits / 8);
    sp.sc_bytes = (uint32_t)((size_t)a.N * sp.G * 2);
    sp.a_bytes = (uint32_t)((size_t)a.M * a.K * 2);
    L.ngc = (a.g >= ck) ? 1 : (int)(ck / a.g);
    L.grid = dim3((unsigned)((sp.NT + p.waves_n - 1) / p.waves_n), (unsigned)p.split_k, (unsigned)p.m_blocks);
    L.block = dim3((unsigned)(64 * p.waves_n * p.waves_k));
    L.lds = sgm.lds;
    L.multi = sgm.multi;
    return L;
}

hipError_t launch_linear(const LinearArgs& a, const LinearPlan& p, hipStream_t st) {
    if (a.zeros && p.path != 1 && p.path != 3) return hipErrorInvalidValue;   // zero points: skinny and wide kernels only
    if (p.path == 3) return launch_linear_wide(a, p, st);
    if (p.path == 4) return launch_linear_tile(a, p, st);
    const SkinnyLaunch L = prepare_skinny(a, p);
    hipError_t e;
    if (a.zeros) {
        if (p.path != 1 || p.prefetch != 1 || p.m_rows16 != 1) return hipErrorInvalidValue;
        e = (a.bits == 4) ? launch_skinny_zp<4>(L.sp, L.ngc, L.multi, L.grid, L.block, L.lds, st)
                          : launch_skinny_zp<8>(L.sp, L.ngc, L.multi, L.grid, L.block, L.lds, st);
    } else if (p.path == 2) {
        e = (a.bits == 4) ? launch_dot<4>(L.sp, L.ngc, L.grid, L.block, L.lds, st) : launch_dot<8>(L.sp, L.ngc, L.grid, L.block, L.lds, st);
    } else {
        e = (a.bits == 4) ? launch_skinny<4>(L.sp, L.ngc, p.prefetch, L.multi, p.m_rows16, L.grid, L.block, L.lds, st)
                          : launch_skinny<8>(L.sp, L.ngc, p.prefetch, L.multi, p.m_rows16, L.grid, L.block, L.lds, st);
    }
    if (e != hipSuccess) return e;
    if (p.split_k > 1) e = launch_splitk_reduce(a.workspace, L.sp.C, a.M * a.N, p.split_k, st);
    return e;
}

template <int BITS, int NGC>
static void launch_grouped_inst(const GroupedParams& gp, bool multi, unsigned blocks, unsigned threads, size_t lds,
                                hipStream_t st) {
    if constexpr (NGC <= Geom<BITS>::NM) {
        if (multi) {
            allow_large_lds(skinny_grouped_kernel<BITS, NGC, true>);
            hipLaunchKernelGGL((skinny_grouped_kernel<BITS, NGC, true>), dim3(blocks), dim3(threads), lds, st, gp);
        } else {
            allow_large_lds(skinny_grouped_kernel<BITS, NGC, false>);
            hipLaunchKernelGGL((skinny_grouped_kernel<BITS, NGC, false>), dim3(blocks), dim3(threads), lds, st, gp);
        }
    }
}

template <int BITS>
static hipError_t launch_grouped_bits(const GroupedParams& gp, int ngc, bool multi, unsigned blocks, unsigned threads,
                                      size_t lds, hipStream_t st) {
    switch (ngc) {
        case 1: launch_grouped_inst<BITS, 1>(gp, multi, blocks, threads, lds, st); break;
        case 2: launch_grouped_inst<BITS, 2>(gp, multi, blocks, threads, lds, st); break;
        case 4: launch_grouped_inst<BITS, 4>(gp, multi, blocks, threads, lds, st); break;
        case 8: launch_grouped_inst<BITS, 8>(gp, multi, blocks, threads, lds, st); break;
        case 16: launch_grouped_inst<BITS, 16>(gp, multi, blocks, threads, lds, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Independent problems: those whose plan is a plain skinny launch (no K split across workgroups, one row block,
// default prefetch) are bucketed by (bits, groups per chunk, workgroup size, staging mode) and every bucket goes
// out as grouped launches of up to kMaxGroup problems; the rest are launched one by one.
hipError_t launch_linear_grouped(const LinearArgs* args, const LinearPlan* plans, int n, hipStream_t st) {
    std::vector<char> done((size_t)n, 0);
    std::vector<SkinnyLaunch> prep((size_t)n);
    std::vector<char> eligible((size_t)n, 0);
    for (int i = 0; i < n; ++i) {
        const LinearPlan& p = plans[i];
        if (p.path != 1 || p.split_k != 1 || p.m_blocks != 1 || p.prefetch != 1 || p.m_rows16 != 1) continue;
        prep[i] = prepare_skinny(args[i], p);
        eligible[i] = 1;
    }
    for (int i = 0; i < n; ++i) {
        if (done[i]) continue;
        if (!eligible[i]) {
            hipError_t e = launch_linear(args[i], plans[i], st);
            if (e != hipSuccess) return e;
            done[i] = 1;
            continue;
        }
        GroupedParams gp;
        gp.n = 0;
        gp.first_block[0] = 0;
        size_t lds = 0;
        for (int j = i; j < n && gp.n < kMaxGroup; ++j) {
            if (done[j] || !eligible[j] || args[j].bits != args[i].bits || prep[j].ngc != prep[i].ngc ||
                prep[j].block.x != prep[i].block.x || prep[j].multi != prep[i].multi)
                continue;
            gp.p[gp.n] = prep[j].sp;
            gp.first_block[gp.n + 1] = gp.first_block[gp.n] + (int)prep[j].grid.x;
            lds = prep[j].lds > lds ? prep[j].lds : lds;
            ++gp.n;
            done[j] = 1;
        }
        const hipError_t e = (args[i].bits == 4)
            ? launch_grouped_bits<4>(gp, prep[i].ngc, prep[i].multi, (unsigned)gp.first_block[gp.n], prep[i].block.x, lds, st)
            : launch_grouped_bits<8>(gp, prep[i].ngc, prep[i].multi, (unsigned)gp.first_block[gp.n], prep[i].block.x, lds, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_splitk_reduce(const float* workspace, void* C_fp16, int64_t MN, int split_k, hipStream_t st) {
    dim3 rgrid((unsigned)((MN / 4 + 255) / 256)), rblock(256);
    half_t* C = static_cast<half_t*>(C_fp16);
    switch (split_k) {
        case 2: hipLaunchKernelGGL(splitk_reduce_kernel<2>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 3: hipLaunchKernelGGL(splitk_reduce_kernel<3>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 4: hipLaunchKernelGGL(splitk_reduce_kernel<4>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 5: hipLaunchKernelGGL(splitk_reduce_kernel<5>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 6: hipLaunchKernelGGL(splitk_reduce_kernel<6>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 7: hipLaunchKernelGGL(splitk_reduce_kernel<7>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        case 8: hipLaunchKernelGGL(splitk_reduce_kernel<8>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
        default: hipLaunchKernelGGL(splitk_reduce_kernel<0>, rgrid, rblock, 0, st, workspace, C, MN, split_k); break;
    }
    return hipGetLastError();
}

}  // namespace rtn
