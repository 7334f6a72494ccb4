/*
 * rtn.h -- C ABI of the MI355X (gfx950) library for weight-only round-to-nearest (RTN)
 * quantised linear layers: the load-time quantise-and-pack pass and the fused
 * dequantise-GEMM used in token generation, plus the selective-precision dispatch.
 *
 * Paper: "Is (Selective) Round-To-Nearest Quantization All You Need?" (arXiv 2505.15909).
 * Each entry point cites the passage that defines the operation it performs.
 *
 * General conventions
 *   - Every pointer named dev_* is DEVICE memory (HIP global memory of the current device);
 *     everything else is host memory.  The caller owns every buffer.  Unless an entry says
 *     otherwise the library allocates nothing, frees nothing and never synchronises: all
 *     work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and is complete when that stream reaches the point after the call.
 *   - All device pointers must be 16-byte aligned.
 *   - Every call validates its arguments on the host before launching anything and
 *     returns an rtn_status; nothing aborts and nothing throws.  A HIP launch failure is
 *     reported as RTN_ERR_HIP.
 *   - Inputs must be finite fp16 values (NaN / Inf give unspecified results).
 *   - Shapes: W is [N, K] (N output channels, K input channels, row-major), activations
 *     A are [M, K] row-major, outputs C are [M, N] row-major, all IEEE binary16.
 *     N % 16 == 0.  K % 512 == 0 for 4-bit, K % 256 == 0 for 8-bit (one k-chunk of the
 *     GEMM kernels).  group_size g: g == K (or g <= 0) means one scale per output channel;
 *     otherwise g must be 32, 64, 128, 256, 512 or a multiple of 512 dividing K for 4-bit and 32, 64,
 *     128, 256 or a multiple of 256 dividing K for 8-bit (the paper uses 128 and per-channel; the
 *     smaller groups of Section 2.2's discussion run on the skinny kernel at every M).
 *   - Size limits of the GEMM entry points (the kernels address each tensor with 32-bit byte offsets): packed
 *     weights N*K*bits/8 and activations M*K*2 must each stay below 0x7FFF0000 bytes (2 GiB - 64 KiB), else
 *     RTN_ERR_SHAPE; M <= 2^20; N <= 2^30; K < 2^23 (group indices come from a multiply-high division that is
 *     exact below that).
 *   - Scales are fp16 [N, K/g] row-major (group j of row n covers columns j*g .. j*g+g-1):
 *     the sub-channel grouping of Section 2.2.
 *
 * Packed weight layout (layout version 1; Section 5: weights are reshuffled once at load
 * into the layout the kernel expects -- this one is designed for gfx950, not Marlin's):
 *   The code matrix is cut into tiles of 16 rows x TK columns, TK = 128 (4-bit) or
 *   64 (8-bit); a tile is 1024 bytes; tiles are stored row-tile-major [N/16][K/TK].
 *   Inside a tile the 16-byte chunk number l (0..63; one per wavefront lane, so a
 *   wavefront reads a tile with one fully coalesced 16-byte-per-lane load) belongs to row
 *   l % 16 and column-quarter kq = l / 16.
 *     4-bit: the chunk is four little-endian 32-bit words t = 0..3; word t holds the 8
 *            codes of columns 32 t + 8 kq + e (e = 0..7), each stored as q + 8 in nibble
 *            number {0,4,1,5,2,6,3,7}[e] (nibble p = bits 4p..4p+3), the order in which a
 *            two-at-a-time mask-and-or unpack produces them.
 *     8-bit: chunk byte 8 t + e (t = 0..1, e = 0..7) holds column 32 t + 8 kq + e as q + 128.
 *   Each (lane, word) therefore carries the 8 consecutive-k values one lane feeds to one
 *   16x16x32 fp16 MFMA.
 */
#ifndef RTN_H_
#define RTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RTN_OK = 0,
    RTN_ERR_NULL = 1,      /* a required pointer is NULL */
    RTN_ERR_BITS = 2,      /* bits is not 4 or 8 */
    RTN_ERR_GROUP = 3,     /* group_size not supported for this K / bits */
    RTN_ERR_SHAPE = 4,     /* M, N or K not supported (see conventions) */
    RTN_ERR_ALIGN = 5,     /* a device pointer is not 16-byte aligned */
    RTN_ERR_WORKSPACE = 6, /* workspace too small for the plan (an explicit split_k, or the small-batch kernel's own) */
    RTN_ERR_CONFIG = 7,    /* explicit kernel configuration invalid for this problem */
    RTN_ERR_HIP = 8        /* the HIP runtime reported an error at launch */
} rtn_status;

/* Scale rule flags of rtn_quantize.  Eq. 2 of Section 2.2 defines S = 2 max|r| / (2^b - 1)
 * = max|r| / (2^(b-1) - 0.5); the default of this library is S = max|r| / (2^(b-1) - 1),
 * under which the group maximum maps exactly onto +-(2^(b-1) - 1) and no code is clamped. */
enum { RTN_SCALE_QMAX = 0, RTN_SCALE_EQ2 = 1 };

/* Horizontal selection policies of Section 4.1. */
enum { RTN_POLICY_FIRST = 0, RTN_POLICY_LAST = 1, RTN_POLICY_MIDDLE = 2 };

const char* rtn_status_str(rtn_status s);
int rtn_layout_version(void);

/* Sizes in bytes of the buffers the caller must provide; 0 if the arguments are invalid.
 * qweight: N*K*bits/8.  scales: N*(K/g)*2.  workspace (rtn_linear, rtn_layer_forward):
 * fp32 split-K partial sums; an upper bound over every configuration the library may
 * choose for this problem; never more than 16 MiB up to 63 rows.  From 64 rows the
 * chosen plan may split K further to fill the compute units (never more than 64 MiB up
 * to 127 rows, 256 MiB above). */
size_t rtn_qweight_nbytes(int64_t N, int64_t K, int bits);
size_t rtn_scales_nbytes(int64_t N, int64_t K, int group_size);
size_t rtn_workspace_nbytes(int64_t M, int64_t N, int64_t K, int bits, int group_size);

/* Load-time RTN quantise-and-pack (Section 2.2, Eq. 1 and Eq. 2, applied per group of g
 * consecutive input columns of every output row; Section 5: done once per weight tensor
 * while loading).  For every group: amax = max|w|; S = fp16(amax / D) with D per `flags`;
 * q = clamp(round_half_even(w / S), -2^(b-1), 2^(b-1)-1), with S the stored fp16 value;
 * a group whose S is zero gets all-zero codes.  Results are bit-exact and deterministic.
 *   dev_W        in   fp16 [N, K]
 *   dev_qweight  out  rtn_qweight_nbytes() bytes, packed layout above
 *   dev_scales   out  fp16 [N, K/g]
 */
rtn_status rtn_quantize(const void* dev_W, int64_t N, int64_t K, int bits, int group_size, int flags,
                        void* dev_qweight, void* dev_scales, void* stream);

/* Load-time pipeline (Sections 1 and 5: a model is quantised on the fly while it is loaded, shard by shard, so the
 * 16-bit model never has to fit the GPU): RTN-quantise a weight tensor that lives in HOST memory.  Shards of
 * rows_per_shard rows (a multiple of 16) are copied into two device staging buffers on `copy_stream` while the previous
 * shard is quantised on `stream`; results are identical to rtn_quantize on the whole tensor.
 *   host_W        in   fp16 [N, K] in host memory; pinned (hipHostMalloc / torch pin_memory) for the copies to overlap
 *   dev_staging   scratch, >= rtn_quantize_host_staging_nbytes(K, rows_per_shard) = 2 shards of fp16 rows
 *   stream, copy_stream   two different streams; the call returns after enqueueing, the packed tensor is complete when
 *                 `stream` reaches the point after the call.  Creates and destroys five events per call (no device memory). */
size_t rtn_quantize_host_staging_nbytes(int64_t K, int64_t rows_per_shard);
rtn_status rtn_quantize_from_host(const void* host_W, int64_t N, int64_t K, int bits, int group_size, int flags,
                                  void* dev_qweight, void* dev_scales, void* dev_staging, size_t staging_nbytes,
                                  int64_t rows_per_shard, void* stream, void* copy_stream);

/* Fused dequantise-GEMM of the weight-only quantised linear layer (Sections 2.3 and 5:
 * 16-bit activations times 4- or 8-bit weights, W4A16 / W8A16, for the small batches of
 * token generation):  C[m, n] = fp16( sum_k A[m, k] * q[n, k] * S[n, k / g] ), products and
 * sums in fp32 (codes enter the matrix cores exactly; the scale multiplies fp32 group
 * partial sums).  Any M >= 1; the path (wavefront-level skinny kernel with split-K for
 * small M, wider MFMA tiles for larger M) is chosen from M, N, K; from 128 rows a call may
 * issue the tile kernel twice (full rounds of workgroups, then the last rows with K split).
 * Deterministic: the same inputs with the same workspace size give the same output bits
 * (split-K partials are summed in a fixed order).
 *   dev_A          in   fp16 [M, K]
 *   dev_qweight    in   packed codes from rtn_quantize
 *   dev_scales     in   fp16 [N, K/g]
 *   dev_C          out  fp16 [M, N]
 *   dev_workspace  scratch, rtn_workspace_nbytes(M, N, K, bits, g) bytes for the plan the library
 *                  prefers (from 17 rows, with less or NULL it splits K less: slower, not an error); contents
 *                  undefined before and after; calls that overlap in time need distinct workspaces
 */
rtn_status rtn_linear(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                      int64_t N, int64_t K, int bits, int group_size, void* dev_C,
                      void* dev_workspace, size_t workspace_nbytes, void* stream);

/* Explicit kernel configuration for rtn_linear_ex (tuning sweeps and tests of every path).
 * A zeroed struct means "choose automatically", field by field. */
typedef struct {
    int path;      /* 0 auto, 1 MFMA skinny kernel, 2 vector-ALU dot-product kernel (M <= 4), 3 wide MFMA kernel
                      (group_size a multiple of 128; uses split_k, m_rows16 = 2..4, n_tiles16 and waves_n = 4, 8 or -- with
                      n_tiles16 = 1 -- 16 wavefronts per workgroup; also m_rows16 = 8 with n_tiles16 = 2 and waves_n = 8:
                      128 rows per workgroup, weights scaled in fp16 before the MFMA as in path 4, chosen automatically
                      for 128 and more rows on large 4-bit matrices below the tile kernel's range), 4 tile kernel: 128 x 256 or
                      256 x 256 output tiles, weights dequantised to fp16 in LDS (group_size a multiple of 128; uses split_k and
                      m_rows16 = 4 or 8 for the tile height, 0 = chosen from M) */
    int prefetch;  /* k-chunks (4 KiB each) a wavefront keeps in flight: 1, 2 or 4 */
    int waves_n;   /* wavefronts of a workgroup along N (share the staged activations): 1 .. 16 */
    int waves_k;   /* wavefronts of a workgroup along K (in-workgroup split-K): 1 .. 16; waves_n * waves_k <= 16 */
    int split_k;   /* workgroups along K (global split-K, reduced through the workspace) */
    int m_rows16;  /* 16-row activation blocks each wavefront multiplies per weight tile: 1, 2 or 4 (path 3: 2, 3, 4, 8) */
    int n_tiles16; /* path 3: 16-column weight tile-rows per wavefront (share each activation operand): 1, 2 or 4;
                      m_rows16 * n_tiles16 <= 8 (or 8 x 2) */
} rtn_linear_cfg;

rtn_status rtn_linear_ex(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                         int64_t N, int64_t K, int bits, int group_size, void* dev_C,
                         void* dev_workspace, size_t workspace_nbytes, void* stream,
                         const rtn_linear_cfg* cfg);

/* Reports the configuration rtn_linear would use (host only, launches nothing). */
rtn_status rtn_linear_query(int64_t M, int64_t N, int64_t K, int bits, int group_size, rtn_linear_cfg* out);

/* Host-only checks, nothing is launched and no pointer is needed.  rtn_problem_status: the status every entry point
 * gives for this (N, K, bits, group_size) before it looks at anything else.  rtn_linear_validate: the status
 * rtn_linear_ex would give for this problem, configuration (NULL = automatic) and workspace size once its pointers
 * have passed (shape, group, configuration and workspace checks; RTN_OK means the launch would be issued). */
rtn_status rtn_problem_status(int64_t N, int64_t K, int bits, int group_size);
rtn_status rtn_linear_validate(int64_t M, int64_t N, int64_t K, int bits, int group_size, size_t workspace_nbytes,
                               const rtn_linear_cfg* cfg);

/* rtn_linear for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments, results and plan as rtn_linear with a
 * workspace of rtn_workspace_nbytes() bytes, but the split-K partial sums go to a fixed 16 MiB device array inside
 * the library (one copy per GPU, held until the process ends) instead of a caller's buffer; the call allocates and
 * frees nothing.  Problems whose rtn_workspace_nbytes() exceeds 16 MiB (only possible from 64 rows) are refused
 * with RTN_ERR_WORKSPACE: use rtn_linear with a workspace for those.  All calls on one GPU share that array, so
 * calls that overlap in time on one GPU (different streams, concurrently replayed graphs) race; calls ordered on a
 * stream are safe.  The first call on a device looks up the array's address (hipGetSymbolAddress); make it before
 * capturing a graph. */
rtn_status rtn_linear_noalloc(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                              int64_t N, int64_t K, int bits, int group_size, void* dev_C, void* stream);

/* Test / debug hook: packed codes -> int8 [N, K] row-major (the inverse of the layout). */
rtn_status rtn_unpack(const void* dev_qweight, int64_t N, int64_t K, int bits, void* dev_codes_i8, void* stream);

/* Dequantise to 16 bit: W'[n, k] = fp16(q[n, k] * S[n, k / g]) -- the first half of the
 * large-input path of Section 5 (dequantise, then a dense 16-bit GEMM). */
rtn_status rtn_dequantize(const void* dev_qweight, const void* dev_scales, int64_t N, int64_t K, int bits,
                          int group_size, void* dev_W_fp16, void* stream);

/* Dense 16-bit GEMM, the second half of the large-input path of Section 5:
 *   C[m, n] = fp16( sum_k A[m, k] * W[n, k] ), fp32 accumulation on the matrix cores.
 *   dev_A fp16 [M, K]; dev_W_fp16 fp16 [N, K] row-major (what rtn_dequantize writes); dev_C fp16 [M, N].
 * K % 128 == 0, N % 16 == 0.  dev_workspace may be NULL (no split-K); otherwise it may be used for split-K partials
 * ([split][M][N] fp32, as many splits as fit) when M and N give too few 128 x 256 output tiles for the compute units. */
rtn_status rtn_gemm_fp16(const void* dev_A, int64_t M, const void* dev_W_fp16, int64_t N, int64_t K, void* dev_C,
                         void* dev_workspace, size_t workspace_nbytes, void* stream);

/* The dual-path forward of Section 5 for inputs with many rows: dequantise the weights to 16 bit into the
 * caller's temporary buffer, then run the dense GEMM.  dev_W_tmp must hold rtn_dense_weight_nbytes(N, K) =
 * 2 N K bytes; its contents afterwards are the dequantised weights.  Same result contract as rtn_linear (each
 * weight is rounded to fp16 once after scaling, inside the layer's tolerance). */
size_t rtn_dense_weight_nbytes(int64_t N, int64_t K);
rtn_status rtn_linear_dense(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                            int64_t N, int64_t K, int bits, int group_size, void* dev_C, void* dev_W_tmp,
                            size_t w_tmp_nbytes, void* dev_workspace, size_t workspace_nbytes, void* stream);

/* One linear module of a Transformer layer with its own precision (Section 4: each of the
 * four linear modules of a layer may be kept at 8 bit while the rest is at 4 bit). */
typedef struct {
    const void* dev_A;        /* fp16 [M, K] */
    int64_t M;
    const void* dev_qweight;
    const void* dev_scales;
    int64_t N, K;
    int bits;                 /* 4 or 8 */
    int group_size;
    void* dev_C;              /* fp16 [M, N] */
} rtn_module;

/* Selective-precision dispatch (Section 4.3, Section 5: RTN-~5 / RTN-~6 models mix 4- and
 * 8-bit modules): runs the n_mods modules in order on `stream`, each with the kernel
 * instantiation of its own (bits, group_size).  The workspace must cover the largest
 * rtn_workspace_nbytes() of the modules; it is reused, which is safe because the launches
 * are ordered on one stream.  Stops at, and returns, the first error. */
rtn_status rtn_layer_forward(const rtn_module* mods, int n_mods, void* dev_workspace,
                             size_t workspace_nbytes, void* stream);

/* ---- Asymmetric variant (the remark after Eq. 1 in Section 2.2: an integer zero point Z is
 * subtracted from the result of Int()).  The paper gives no more than that; this library
 * takes, per group of g columns of a row:
 *   [alpha, beta] = [min(min w, 0), max(max w, 0)]      (zero is always a level)
 *   S = fp16((beta - alpha) / (2^b - 1)), the exact quotient rounded once (as for the symmetric scale)
 *   Z = clamp(rne(alpha / S), -(2^b - 1), 0) + 2^(b-1)  (alpha goes to the lowest code)
 *   q = clamp(rne(w / S) - Z, -2^(b-1), 2^(b-1) - 1)    (ties on w / S, before Z)
 * and the dequantised weight is S * (q + Z).  S == 0 gives Z = 2^(b-1), q = -2^(b-1).
 * Codes use the same packed layout (rtn_unpack returns q); dev_zeros is fp16 [N, K/g]
 * holding the integers Z; sizes as for the scales (rtn_scales_nbytes).  Group sizes, shapes,
 * alignment and error behaviour as for rtn_quantize / rtn_dequantize / rtn_linear.
 * rtn_linear_asym runs the small-batch kernel up to 16 rows and the wide MFMA kernel above (group
 * sizes that are multiples of 128; other group sizes go 16 rows at a time and re-read the weights);
 * for thousands of rows dequantise once with rtn_dequantize_asym and call rtn_gemm_fp16. */
rtn_status rtn_quantize_asym(const void* dev_W, int64_t N, int64_t K, int bits, int group_size,
                             void* dev_qweight, void* dev_scales, void* dev_zeros, void* stream);
rtn_status rtn_dequantize_asym(const void* dev_qweight, const void* dev_scales, const void* dev_zeros,
                               int64_t N, int64_t K, int bits, int group_size, void* dev_W_fp16,
                               void* stream);
/*   C[m, n] = fp16( sum_k A[m, k] * S[n, k/g] * (q[n, k] + Z[n, k/g]) ), fp32 accumulation. */
rtn_status rtn_linear_asym(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                           const void* dev_zeros, int64_t N, int64_t K, int bits, int group_size,
                           void* dev_C, void* dev_workspace, size_t workspace_nbytes, void* stream);

/* Grouped call for modules that do not depend on one another: the experts of a
 * mixture-of-experts layer, each with its own weight matrix, its own rows of activations
 * and -- the per-expert precision that Section 6 (Discussion) proposes, with the Mixtral
 * 8x22B remark of the Limitations section -- its own bits; or projections that read the
 * same input.  Same arguments and validation as
 * rtn_layer_forward, but nothing is launched unless every module passes, the launch order
 * is unspecified, and modules with M <= 16 and the same (bits, group size) class are merged,
 * up to 16 at a time, into single grids whose workgroups each serve one module, so that one
 * launch streams all their weights.  No dev_C may overlap any module's dev_A.  Results are
 * those of rtn_linear with the plan rtn_grouped_forward picks (planned for the summed size),
 * which may differ from the single call's in summation order only. */
rtn_status rtn_grouped_forward(const rtn_module* mods, int n_mods, void* dev_workspace,
                               size_t workspace_nbytes, void* stream);

/* Measurement hook (Section 1: token generation is bound by the weight bytes that must be read): a plain read
 * kernel that streams dev_buf once, 16 bytes per lane and load, kib_per_wavefront (1..64) consecutive KiB per
 * wavefront, and computes nothing.  Its time on a buffer the size of a packed weight matrix is the read-stream ceiling
 * that the fused kernels are reported against, beside the published HBM peak.  nbytes a multiple of 1024; dev_buf
 * 16-byte aligned; dev_sink: 4 bytes of device memory (never written for any real data). */
rtn_status rtn_bench_read_stream(const void* dev_buf, size_t nbytes, int kib_per_wavefront, void* dev_sink,
                                 void* stream);

/* Hybrid selection rule of Section 4.3: bits of module `module_id` (1 = QKV projection,
 * 2 = attention output projection, 3 and 4 = feed-forward, numbering of Section 4.2) of
 * 0-based `layer` when X layers chosen by `policy` (first / last / middle, Section 4.1)
 * keep the modules in `module_mask` (bit i-1 set = module i) at 8 bit and everything else
 * is 4 bit.  Returns 4 or 8, or -1 on invalid arguments.  Host only. */
int rtn_plan_bits(int layer, int n_layers, int module_id, int policy, int X, unsigned module_mask);

/* Average bits per weight of such a plan (Section 4.3: a quarter / a half of the layers at 8 bit average 5 / 6 bits);
 * module_params[i] = weights of module i+1 in one layer.  Returns -1 on invalid arguments. */
double rtn_plan_effective_bits(int n_layers, const int64_t module_params[4], int policy, int X,
                               unsigned module_mask);

#ifdef __cplusplus
}
#endif
#endif /* RTN_H_ */
