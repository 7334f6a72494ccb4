// Host-side interfaces between the C-ABI translation unit and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtn {

constexpr size_t kMaxLdsBytes = 160 * 1024;   // LDS of one gfx950 compute unit, usable by one workgroup

// Resolved launch configuration of the fused dequantise-GEMM.
struct LinearPlan {
    int path;       // 1 = MFMA skinny kernel, 2 = vector-ALU dot kernel, 3 = wide MFMA kernel (larger batches),
                    // 4 = tile kernel, 128 or 256 rows x 256 columns per workgroup (matrix-core bound batches)
    int prefetch;   // k-chunks in flight per wavefront (register buffers): 1, 2 or 4
    int waves_n;    // wavefronts along N per workgroup
    int waves_k;    // wavefronts along K per workgroup
    int split_k;    // workgroups along K
    int m_rows16;   // 16-row activation blocks per wavefront: 1, 2 or 4 (prefetch must be 1 above 1)
    int m_blocks;   // activation blocks of 16 * m_rows16 rows (grid.z)
    int n_tiles16;  // path 3: 16-column weight tile-rows per wavefront: 1, 2 or 4
};

struct LinearArgs {
    const void* A;
    const void* qweight;
    const void* scales;
    void* C;
    float* workspace;
    int64_t M, N, K, g;
    int bits;
    const void* zeros = nullptr;   // fp16 [N, K/g] integer zero points (asymmetric variant; skinny and wide kernels) or null
};

hipError_t launch_quantize(const void* W, int64_t N, int64_t K, int bits, int64_t g, float divisor,
                           void* qweight, void* scales, hipStream_t st);
// Asymmetric variant: codes, fp16 scales and fp16 integer zero points Z, dequantised weight S (q + Z).
hipError_t launch_quantize_asym(const void* W, int64_t N, int64_t K, int bits, int64_t g, void* qweight, void* scales,
                                void* zeros, hipStream_t st);
// zeros: null for the symmetric variant.
hipError_t launch_unpack(const void* qweight, const void* scales, int64_t N, int64_t K, int bits, int64_t g,
                         bool dequant, void* out, hipStream_t st, const void* zeros = nullptr);
hipError_t launch_linear(const LinearArgs& a, const LinearPlan& p, hipStream_t st);
// n independent problems with resolved plans: compatible skinny-kernel launches are merged into grouped launches.
hipError_t launch_linear_grouped(const LinearArgs* args, const LinearPlan* plans, int n, hipStream_t st);
// Path 3 (wide MFMA kernel): plan check (group size a multiple of 128, 2-4 row blocks, 1/2/4 tile-rows, at most 8 blocks) and launch.
bool wide_plan_valid(const LinearArgs& a, const LinearPlan& p);
hipError_t launch_linear_wide(const LinearArgs& a, const LinearPlan& p, hipStream_t st);
// Path 4 (tile kernel, weights dequantised into LDS): plan check (group size a multiple of 128) and launch.
bool tile_plan_valid(const LinearArgs& a, const LinearPlan& p);
hipError_t launch_linear_tile(const LinearArgs& a, const LinearPlan& p, hipStream_t st);
// Dense fp16 GEMM C[M,N] = A[M,K] W[N,K]^T with the same tile kernel (K a multiple of 128); split_k > 1 goes
// through the fp32 workspace [split_k][M][N].
hipError_t launch_gemm_fp16(const void* A, const void* W, void* C, float* workspace, int64_t M, int64_t N, int64_t K,
                            int split_k, hipStream_t st);
// Sums split_k fp32 partial outputs [split_k][MN] in a fixed order into fp16 C (MN a multiple of 16).
hipError_t launch_splitk_reduce(const float* workspace, void* C_fp16, int64_t MN, int split_k, hipStream_t st);

// LDS bytes the skinny kernel needs for a plan (staged activation slice incl. the zero row, or the
// in-workgroup split-K reduction buffer, whichever is larger).
size_t linear_lds_bytes(const LinearArgs& a, const LinearPlan& p);
// Whether the plan's activation staging fits the LDS limit and the per-thread staging registers.
bool linear_plan_fits(const LinearArgs& a, const LinearPlan& p, size_t lds_limit);

}  // namespace rtn
