// Host-only driver for the sanitizer build of the library's planning and validation code (no GPU work: only entry
// points that launch nothing).  Built by tests/test_host_sanitizers.py with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side and run on the CPU; any report makes the run fail.
#include "../../include/rtn.h"
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <initializer_list>

static uint64_t state = 0x2505159091234567ull;
static uint64_t next_u64() {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return state;
}
static int64_t pick(int64_t lo, int64_t hi) { return lo + (int64_t)(next_u64() % (uint64_t)(hi - lo + 1)); }

int main() {
    long calls = 0, ok = 0;
    const int64_t Ms[] = {1, 2, 3, 4, 5, 8, 9, 15, 16, 17, 31, 32, 33, 48, 49, 64, 65, 96, 100, 127, 128, 129, 144, 191, 192,
                          256, 300, 511, 1000, 1024, 2048, 4096, 16384, 100000, 1 << 20};
    const int groups[] = {0, -1, 32, 64, 128, 256, 512, 1024, 2048, 96, 100, 16};
    // the paper's Llama shapes, small ones, and random ones (valid and invalid mixed)
    int64_t shapes[200][2];
    int ns = 0;
    const int64_t fixed[][2] = {{4096, 6144}, {4096, 4096}, {4096, 28672}, {14336, 4096}, {8192, 10240}, {8192, 8192}, {8192, 57344},
                                {28672, 8192}, {16384, 18432}, {16384, 16384}, {16384, 106496}, {53248, 16384}, {2048, 3072},
                                {2048, 2048}, {2048, 16384}, {8192, 2048}, {3072, 5120}, {3072, 3072}, {8192, 3072}, {512, 16},
                                {256, 16}, {1024, 1048576}, {8388096, 16}, {8388608, 16}, {500, 64}, {512, 60}, {0, 16}, {512, 0}};
    for (auto& f : fixed) { shapes[ns][0] = f[0]; shapes[ns][1] = f[1]; ++ns; }
    while (ns < 200) { shapes[ns][0] = pick(1, 120) * 256; shapes[ns][1] = pick(1, 7000) * 16; ++ns; }
    for (int si = 0; si < ns; ++si) {
        const int64_t K = shapes[si][0], N = shapes[si][1];
        for (int bits : {4, 8, 5}) {
            for (int g : groups) {
                (void)rtn_qweight_nbytes(N, K, bits);
                (void)rtn_scales_nbytes(N, K, g);
                const rtn_status ps = rtn_problem_status(N, K, bits, g);
                ++calls;
                for (int64_t M : Ms) {
                    const size_t ws = rtn_workspace_nbytes(M, N, K, bits, g);
                    rtn_linear_cfg q = {};
                    const rtn_status qs = rtn_linear_query(M, N, K, bits, g, &q);
                    ++calls;
                    const bool too_big = (uint64_t)N * K * bits / 8 >= 0x7FFF0000ull || (uint64_t)M * K * 2 >= 0x7FFF0000ull;
                    if (ps == RTN_OK && too_big) {
                        if (qs != RTN_ERR_SHAPE) { printf("size limit not reported N=%ld K=%ld M=%ld\n", (long)N, (long)K, (long)M); return 1; }
                        continue;
                    }
                    if ((ps == RTN_OK) != (qs == RTN_OK)) { printf("status mismatch N=%ld K=%ld bits=%d g=%d\n", (long)N, (long)K, bits, g); return 1; }
                    if (qs != RTN_OK) continue;
                    // the automatic plan, handed back explicitly, validates within the workspace the size helper promises
                    rtn_status vs = rtn_linear_validate(M, N, K, bits, g, ws, &q);
                    ++calls;
                    if (vs != RTN_OK) { printf("auto plan invalid: M=%ld N=%ld K=%ld bits=%d g=%d status %d\n", (long)M, (long)N, (long)K, bits, g, (int)vs); return 1; }
                    ++ok;
                    vs = rtn_linear_validate(M, N, K, bits, g, 0, nullptr);          // no workspace at all
                    vs = rtn_linear_validate(M, N, K, bits, g, 256, nullptr);
                    // random explicit configurations: any status is fine, a sanitizer report is not
                    for (int t = 0; t < 6; ++t) {
                        rtn_linear_cfg c = {(int)pick(0, 5), (int)pick(0, 5), (int)pick(0, 17), (int)pick(0, 17), (int)pick(0, 20),
                                            (int)pick(0, 9), (int)pick(0, 5)};
                        (void)rtn_linear_validate(M, N, K, bits, g, (size_t)pick(0, 1 << 28), &c);
                        ++calls;
                    }
                }
            }
        }
    }
    // selective-precision bookkeeping
    const int64_t params[4] = {4096 * 6144, 4096 * 4096, 4096 * 28672, 14336 * 4096};
    for (int n_layers : {0, 1, 2, 32, 80, 126})
        for (int policy = -1; policy <= 3; ++policy)
            for (int X = -1; X <= n_layers + 1; X += (n_layers > 8 ? 7 : 1))
                for (unsigned mask = 0; mask <= 17; ++mask) {
                    (void)rtn_plan_effective_bits(n_layers, params, policy, X, mask);
                    for (int layer = -1; layer <= n_layers; layer += (n_layers > 8 ? 5 : 1))
                        for (int mod = 0; mod <= 5; ++mod) (void)rtn_plan_bits(layer, n_layers, mod, policy, X, mask);
                    ++calls;
                }
    for (int s = 0; s <= 8; ++s) (void)rtn_status_str((rtn_status)s);
    (void)rtn_quantize_host_staging_nbytes(4096, 64);
    (void)rtn_dense_weight_nbytes(4096, 4096);
    printf("host sanitizer driver: %ld calls, %ld automatic plans validated\n", calls, ok);
    return ok > 10000 ? 0 : 1;
}
