// C ABI of the library (see include/rtn.h): argument validation, kernel-plan selection,
// selective-precision dispatch.  No device code here.
#include "../../include/rtn.h"
#include "rtn_internal.h"
#include <vector>
#include <algorithm>
#include <cmath>
#include <mutex>

#include <stdlib.h>
#include <string.h>

using rtn::LinearArgs;
using rtn::LinearPlan;

namespace {

constexpr size_t kWorkspaceCap = (size_t)16 << 20;     // split-K partials never exceed this ...
constexpr size_t kWorkspaceCapTall = (size_t)64 << 20; // ... except under the wide kernel's plans from 64 rows (and the tile kernel's)
constexpr int kMaxSplitK = 16;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int chunk_k(int bits) { return bits == 4 ? 512 : 256; }
int tile_k(int bits) { return bits == 4 ? 128 : 64; }

// Normalises group_size (<= 0 or K means per-channel) and checks it.
rtn_status check_problem(int64_t N, int64_t K, int bits, int group_size, int64_t* g_out) {
    if (bits != 4 && bits != 8) return RTN_ERR_BITS;
    if (N <= 0 || K <= 0 || N % 16 != 0 || K % chunk_k(bits) != 0) return RTN_ERR_SHAPE;
    // K < 2^23: the kernels divide k-step and chunk indices by the group length with a multiply-high by
    // floor(2^32 / d) + 1, exact while index * d < 2^32
    if (N > (int64_t)1 << 30 || K >= (int64_t)1 << 23) return RTN_ERR_SHAPE;
    int64_t g = (group_size <= 0) ? K : group_size;
    if (g > K || K % g != 0) return RTN_ERR_GROUP;
    const int ck = chunk_k(bits), tk = tile_k(bits);
    if (g < ck) {                                   // 32, 64, ... up to a k-chunk: a power-of-two number of groups per chunk
        if (g != 32 && g != 64 && g != tk && g != 2 * tk && g != 4 * tk) return RTN_ERR_GROUP;
    } else if (g % ck != 0) {
        return RTN_ERR_GROUP;
    }
    *g_out = g;
    return RTN_OK;
}

size_t workspace_bound(int64_t M, int64_t N) {
    size_t one = (size_t)M * (size_t)N * sizeof(float);
    size_t want = one * kMaxSplitK;
    if (want > kWorkspaceCap) want = kWorkspaceCap;
    if (want < 256) want = 256;
    return (want + 255) & ~(size_t)255;
}

int device_max_lds() {
    static int cached = 0;
    if (cached == 0) {
        int v = 0, dev = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
            cached = v < (int)rtn::kMaxLdsBytes ? v : (int)rtn::kMaxLdsBytes;
        else
            cached = (int)rtn::kMaxLdsBytes;   // no device to ask (host-only planning): the gfx950 figure
    }
    return cached;
}

int round_pow2(int64_t v, int lo, int hi) {
    int p = lo;
    while (p * 2 <= hi && (int64_t)p * 3 / 2 <= v) p *= 2;     // nearest power of two in the log sense
    return p;
}

// Default plan, from configuration sweeps on MI355X.  Short-lived wavefronts at high
// occupancy stream best: a wavefront gets 1-4 k-chunks (4-16 KiB of packed weights) of one tile-row
// and K is split inside the workgroup (reduced through LDS).  With more than two activation rows the
// staged slice grows, so workgroups widen along N (sharing it) and, for long K, K is also split across
// workgroups so that a slice stays a few chunks long; those partials go through the workspace.
// Plan of the wide MFMA kernel for more than 16 rows: the candidate (wavefronts per workgroup, tile-rows per
// wavefront, K splits) with the lowest modelled time.  The model is the larger of three streaming / arithmetic
// times -- activations re-read from L2 once per workgroup column plus the weights, the weights from HBM, the
// MFMA work -- derated by how evenly the workgroups fill the compute units, plus fixed per-launch, per-round and
// split-K reduction costs.  Its constants were fitted to sweeps over the 8B, 70B and 405B shapes at 32-256
// rows, where its choice is within 2 % of the best measured configuration on average (worst case 15 %).
double wide_model_us(int64_t M, int64_t N, int64_t K, int bits, int mb, int wv, int nbw, int s) {
    const double kL2 = 11.26e12, kHbm = 6.96e12, kMfma = 1.02e15, kSmallTile = 0.767, kFix = 2e-6, kRound = 1.5e-6;
    const double kReduce0 = 2.5e-6, kReduceBw = 4.55e12, kUtilExp = 0.662;
    const int64_t rows = 16 * mb, ZB = (M + rows - 1) / rows, n_wg = 16 * nbw * wv, XB = (N + n_wg - 1) / n_wg;
    const int64_t wgs = XB * ZB * s, slots = 256 * (wv == 4 ? 3 : 1);
    const int64_t rounds = (wgs + slots - 1) / slots;
    const double util = (double)wgs / (double)(rounds * slots);
    const double Mp = (double)(ZB * rows), wbytes = (double)N * K * bits / 8.0;
    const double t_l2 = (2.0 * Mp * K * XB + wbytes * std::sqrt((double)ZB)) / kL2;
    const double t_hbm = wbytes * 1.03 / kHbm;
    const double t_mfma = 2.0 * Mp * N * K / (kMfma * (nbw * mb >= 8 ? 1.0 : kSmallTile));
    double t = std::max(t_l2, std::max(t_hbm, t_mfma)) / std::pow(util, kUtilExp) + kFix + rounds * kRound;
    if (s > 1) t += kReduce0 + 2.0 * s * M * N * 4.0 / kReduceBw;
    return t * 1e6;
}

void wide_plan(int64_t M, int64_t N, int64_t K, int bits, LinearPlan* p) {
    p->path = 3;
    p->m_rows16 = M <= 32 ? 2 : (M <= 48 ? 3 : 4);
    // 48-row blocks above 64 rows where they save a fifth of the padded rows (65-96 and 129-144 rows: 96 against 128,
    // 144 against 192): 3-20 % faster there on the 8B, 70B and 405B shapes (a 48-row block is 10-15 % slower per row).
    // Workgroup shape and K split are still the ones modelled for 64-row blocks: the model's own choice for 48-row
    // blocks splits K too little (measured: 9-14 % slower on six of the shapes).
    const bool blocks48 = M > 64 && ((M + 47) / 48) * 48 * 5 <= ((M + 63) / 64) * 64 * 4;
    p->m_blocks = (int)((M + 16 * p->m_rows16 - 1) / (16 * p->m_rows16));
    p->prefetch = 1; p->waves_k = 1;
    const int64_t KS = K / 128;
    int64_t smax = (int64_t)((M >= 64 ? kWorkspaceCapTall : kWorkspaceCap) / ((size_t)M * N * sizeof(float)));
    if (smax > kMaxSplitK) smax = kMaxSplitK;
    if (smax > KS / 4) smax = KS / 4;
    if (smax < 1) smax = 1;
    // three splits (they fill the compute units where two leave a third idle and four start a second round) compete
    // with the powers of two: 19-34 % faster on the 70B and 405B qkv matrices at 48-128 rows.  Other splits are taken
    // only when the model puts them 5 % ahead: its small preferences for five or six on the 8B shapes cost 2-3 %.
    double best = 1e30, best_any = 1e30;
    LinearPlan any = *p;
    for (int wv = 4; wv <= 16; wv *= 2)
        for (int nbw = 1; nbw <= 4; nbw *= 2) {
            if (p->m_rows16 * nbw > 8 || (wv == 16 && nbw > 1)) continue;
            for (int s = 1; s <= smax; ++s) {
                const double t = wide_model_us(M, N, K, bits, p->m_rows16, wv, nbw, s);
                if (((s & (s - 1)) == 0 || s == 3) && t < best) {
                    best = t;
                    p->waves_n = wv; p->n_tiles16 = nbw; p->split_k = s;
                }
                if (t < best_any) {
                    best_any = t;
                    any.waves_n = wv; any.n_tiles16 = nbw; any.split_k = s;
                }
            }
        }
    if (best_any < 0.95 * best) {
        p->waves_n = any.waves_n; p->n_tiles16 = any.n_tiles16; p->split_k = any.split_k;
    }
    if (blocks48) {
        p->m_rows16 = 3;
        p->m_blocks = (int)((M + 47) / 48);
    }
}

// K splits of the wide kernel's 128-row variant (128 rows x 256 columns per workgroup, one workgroup per compute
// unit): the lowest modelled time over 1, 2, 4, 8 splits that fit 64 MiB of partials.  A workgroup's full-K time is
// its MFMA work at the 4.3 TFLOP/s one compute unit sustains in this kernel; a round of workgroups costs 9 us more
// (start, prologue, epilogue), the reduce launch 4 us plus its traffic at 5 TB/s.  Fitted to sweeps over the 70B and
// 405B shapes at 128-512 rows, where it picks the measured best split or one within 4 % of it.
int tall_wide_split(int64_t M, int64_t N, int64_t K) {
    const int64_t wgs = ((N + 255) / 256) * ((M + 127) / 128);
    const double t1 = 2.0 * 128 * 256 * (double)K / 4.3e12, mn4 = (double)M * N * 4.0;
    int best_s = 1;
    double best = 1e30;
    for (int s = 1; s <= 8; ++s) {
        if (s > 1 && ((size_t)M * N * sizeof(float) * s > kWorkspaceCapTall || K / 128 / s < 4)) break;
        const double rounds = (double)((wgs * s + 255) / 256);
        double t = rounds * (t1 / s + 9e-6);
        if (s > 1) t += 4e-6 + 2.0 * s * mn4 / 5e12;
        if (t < best) { best = t; best_s = s; }
    }
    return best_s;
}

// Tile height (128 or 256 rows) and K split of the fused tile kernel: the pair with the lowest modelled time.  One
// workgroup runs per compute unit, so a launch takes rounds of 256 workgroups; a workgroup advances one 64-column step
// in 0.85 us with a 128-row tile and 1.40 us with a 256-row tile (packed weights) and costs 8 us besides; a split adds
// the reduce launch and the partial sums' trip through the workspace at 4 TB/s.  Splits need not be powers of two: what
// pays is a split that fills the last round (144 tiles: three splits of 72 tall tiles make one round of 216).  Fitted
// to a sweep of splits 1-8 and both heights over the 8B, 70B and 405B shapes whose tiles fill their last round
// to less than 85 %: the pick is within 1 % of the best measured pair on average, where one split and the height rule
// of the launch were 6 % behind (405B qkv at 256 rows: 163 us against 219).
constexpr size_t kWorkspaceCapTile = (size_t)256 << 20;
double tile_plan_choose(int64_t M, int64_t N, int64_t K, int* rows16, int* split_k) {
    const int64_t xb = (N + 255) / 256;
    double best = 1e30;
    *rows16 = 4; *split_k = 1;
    for (int s = 1; s <= 8; ++s) {
        if (s > 1 && ((size_t)M * N * sizeof(float) * s > kWorkspaceCapTile || K / 128 / s < 4)) break;
        for (int h = 4; h <= 8; h += 4) {
            if (h == 8 && M <= 128) continue;
            const int64_t tiles = xb * ((M + 32 * h - 1) / (32 * h));
            const double rounds = (double)((tiles * s + 255) / 256), steps = (double)((K / 64 + s - 1) / s);
            double t = rounds * (steps * (h == 4 ? 0.85 : 1.40) + 8.0);
            if (s > 1) t += 2.5 + (2.0 * s * M * N * 4.0 + 2.0 * M * N) / 4.0e6;
            if (t < best) { best = t; *rows16 = h; *split_k = s; }
        }
    }
    return best;
}

// The tile kernel in two launches: the first rows_first rows (a multiple of 256) as full rounds of workgroups, the
// rest as a launch of its own, which the plan above gives the K split that fills its one round.  Returns rows_first,
// or 0 where one launch is modelled within 7 % of the best pair.  Measured as two calls against one on the qkv shapes:
// 405B at 2048 rows 1044 us against 1236, at 1024 rows 565 against 641; 70B at 2048 rows 324 against 374; 8B at 4096
// rows 208 against 232; no gain (and none modelled) where the tiles fill their rounds.
int64_t tile_two_launches(int64_t M, int64_t N, int64_t K) {
    if (M > 16384) return 0;                                   // many rounds: the last one no longer matters
    int r16, sk;
    const double single = tile_plan_choose(M, N, K, &r16, &sk);
    double best = single * 0.93;
    int64_t rows_first = 0;
    for (int64_t r1 = 256; r1 < M; r1 += 256) {
        const double t = tile_plan_choose(r1, N, K, &r16, &sk) + tile_plan_choose(M - r1, N, K, &r16, &sk);
        if (t < best) { best = t; rows_first = r1; }
    }
    return rows_first;
}

// Plan of the small-batch (skinny) kernel for up to 16 rows: a table of measured configurations on a grid of
// problems -- tile-rows N / 16 from 64 to 8192 and k-chunks per row from 2 to 128, by powers of two and at the 1.5 x
// points between them, 1, 2, 4, 8, 16 rows, both precisions -- plus the linear modules of the Llama 3.1 8B / 70B / 405B and Llama 3.2 1B / 3B
// layers the paper evaluates (Table 1).  Every entry lists its twelve fastest configurations with their slowdown
// against the fastest.  A problem that is in the table takes its entry's ranking; any other one lets its three nearest
// entries (distance in log2 of tile-rows, chunks per row and rows) vote: a configuration's score is the weighted mean
// log slowdown over the three (1.5 x where an entry does not list it), and the best-scored configuration that is valid
// for the problem wins.  On shapes outside the table (tuning/shapes_heldout.txt) the pick is about 1 % behind the best
// measured configuration at the median and within 10 % on nineteen problems out of twenty.
// tuning/plan_sweep.hip measures, tuning/make_plan_table.py writes the table.
constexpr int kPlanEntryConfigs = 12;
struct SkinnyPlanConfig {
    uint8_t wn, wk, split, nb, slow;       // slow: slowdown against the entry's fastest, units of 0.5 %
};
struct SkinnyPlanEntry {
    uint8_t bits;
    uint16_t nt, kc;
    uint8_t m, n;
    SkinnyPlanConfig c[kPlanEntryConfigs];
};
const SkinnyPlanEntry kSkinnyPlanTable[] = {
#include "skinny_plan_table.inc"
};

bool skinny_plan_usable(int64_t M, int64_t N, int64_t K, int bits, const LinearPlan& p, size_t lds_limit) {
    const int64_t KC = K / chunk_k(bits);
    if (p.waves_n < 1 || p.waves_k < 1 || p.waves_n * p.waves_k > 16) return false;
    if (p.split_k < 1 || p.split_k > kMaxSplitK || p.split_k > KC) return false;
    if (p.split_k > 1 && (size_t)M * N * sizeof(float) * p.split_k > kWorkspaceCap) return false;
    LinearArgs a;
    a.M = M; a.N = N; a.K = K; a.bits = bits; a.g = K;
    return rtn::linear_plan_fits(a, p, lds_limit);
}

// Workgroups come in rounds of one per compute unit: a launch of n workgroups keeps the busiest of the 256 compute units
// ceil(n / 256) workgroups long where n / 256 would be the average.  Coarse configurations (few, long-lived workgroups)
// pay for it: 269 workgroups of eight wavefronts take 1.45 x the time of 256.  The table's grid shapes are powers of
// two, the best case, so a configuration's measured slowdown is corrected by this ratio to the power 0.7 (fitted on
// shapes outside the table), entry against problem.
constexpr double kImbalanceExp = 0.7;
constexpr double kWidthStep = 0.3;      // log-time per octave of workgroup width away from a voted configuration
double cu_imbalance(int64_t workgroups) {
    const double avg = (double)workgroups / 256.0;
    return std::ceil(avg) / avg;
}

bool skinny_plan_from_table(int64_t M, int64_t N, int64_t K, int bits, size_t lds_limit, LinearPlan* out) {
    const double fnt = std::log2((double)(N / 16)), fkc = std::log2((double)(K / chunk_k(bits))), fm = std::log2((double)M);
    const int n = (int)(sizeof(kSkinnyPlanTable) / sizeof(kSkinnyPlanTable[0]));
    constexpr int kVoters = 3;
    int near_i[kVoters];
    double near_d[kVoters];
    int found = 0;
    for (int i = 0; i < n; ++i) {
        const SkinnyPlanEntry& e = kSkinnyPlanTable[i];
        if (e.bits != bits) continue;
        const double d = 2.0 * std::fabs(std::log2((double)e.nt) - fnt) + std::fabs(std::log2((double)e.kc) - fkc) +
                         0.5 * std::fabs(std::log2((double)e.m) - fm);
        int pos = found < kVoters ? found : kVoters;             // insertion into the sorted list of the nearest
        while (pos > 0 && d < near_d[pos - 1]) --pos;
        if (pos >= kVoters) continue;
        for (int q = (found < kVoters ? found : kVoters - 1); q > pos; --q) { near_i[q] = near_i[q - 1]; near_d[q] = near_d[q - 1]; }
        near_i[pos] = i; near_d[pos] = d;
        if (found < kVoters) ++found;
    }
    if (found == 0) return false;
    if (near_d[0] < 1e-9) found = 1;                            // the problem itself is in the table: its own ranking
    struct Scored { SkinnyPlanConfig c; double base, score; };
    std::vector<Scored> cand;
    cand.reserve(kVoters * kPlanEntryConfigs * 8);
    const double kMissing = std::log(1.5);
    const int64_t NT = N / 16;
    auto same = [](const SkinnyPlanConfig& a, const SkinnyPlanConfig& b) {
        return a.wn == b.wn && a.wk == b.wk && a.split == b.split && a.nb == b.nb;
    };
    auto imbalance_of = [](int64_t nt, const SkinnyPlanConfig& c) {
        return std::log(cu_imbalance(((nt + c.wn - 1) / c.wn) * c.split));
    };
    for (int v = 0; v < found; ++v) {
        const SkinnyPlanEntry& e = kSkinnyPlanTable[near_i[v]];
        for (int k = 0; k < e.n; ++k) {
            bool seen = false;
            for (size_t q = 0; q < cand.size() && !seen; ++q) seen = same(cand[q].c, e.c[k]);
            if (seen) continue;
            double num = 0.0, den = 0.0;
            for (int u = 0; u < found; ++u) {
                const SkinnyPlanEntry& f = kSkinnyPlanTable[near_i[u]];
                const double w = 1.0 / (near_d[u] + 0.25);
                double ls = kMissing;
                for (int q = 0; q < f.n; ++q)
                    if (same(f.c[q], e.c[k])) {
                        ls = std::min(kMissing, std::log(1.0 + f.c[q].slow / 200.0));
                        break;
                    }
                // the entry's own workgroup-count imbalance is taken out of its measurement ...
                ls -= kImbalanceExp * imbalance_of(f.nt, e.c[k]);
                num += w * ls; den += w;
            }
            // ... and the problem's own put in; ties: the order of the nearer entry
            const double base = num / den;
            cand.push_back({e.c[k], base, base + kImbalanceExp * imbalance_of(NT, e.c[k]) + 1e-9 * (double)cand.size()});
        }
    }
    // Workgroup width follows the problem, not the table: a voted configuration one or two wavefronts deep along K also
    // stands for its neighbours with any other number of wavefronts along N (1 .. 16 / waves_k), scored as itself with
    // the neighbour's workgroup-count imbalance and kWidthStep per octave of width moved.  The table's grid has powers
    // of two of tile-rows, where powers of two of wavefronts always divide evenly; a matrix of, say, 2153 tile-rows
    // is served 25-35 % faster at 16 rows by nine wavefronts (240 workgroups) than by eight (270, a second round on
    // fourteen compute units).  Not applied when the problem itself is in the table.
    if (found > 1) {
        const size_t voted = cand.size();
        for (size_t q = 0; q < voted; ++q) {
            const SkinnyPlanConfig c = cand[q].c;
            if (c.wk > 2 || c.split > 4 || (c.wk == 1 && c.nb == 1 && c.split > 1) || (c.wk == 2 && c.split > 2)) continue;
            for (int w2 = 1; w2 <= 16 / c.wk; ++w2) {
                if (w2 == c.wn || w2 > NT) continue;
                SkinnyPlanConfig c2 = c;
                c2.wn = (uint8_t)w2;
                const double sc = cand[q].base + kImbalanceExp * imbalance_of(NT, c2) +
                                  kWidthStep * std::fabs(std::log2((double)w2 / c.wn)) + 1e-6;
                size_t at = 0;
                while (at < cand.size() && !same(cand[at].c, c2)) ++at;
                if (at < voted) continue;                            // voted on directly
                if (at == cand.size()) cand.push_back({c2, cand[q].base, sc});
                else if (sc < cand[at].score) cand[at].score = sc;
            }
        }
    }
    const int nc = (int)cand.size();
    std::sort(cand.begin(), cand.end(), [](const Scored& a, const Scored& b) { return a.score < b.score; });
    for (int q = 0; q < nc; ++q) {
        LinearPlan p;
        p.path = 1; p.n_tiles16 = 1; p.m_rows16 = 1; p.m_blocks = 1;
        p.prefetch = cand[q].c.nb; p.waves_n = cand[q].c.wn; p.waves_k = cand[q].c.wk; p.split_k = cand[q].c.split;
        while (p.waves_n > 1 && p.waves_n > N / 16) p.waves_n /= 2;
        if (skinny_plan_usable(M, N, K, bits, p, lds_limit)) { *out = p; return true; }
    }
    return false;
}

// force_path: 0 = choose the path, otherwise the default plan of that path.
LinearPlan auto_plan(int64_t M, int64_t N, int64_t K, int bits, int64_t g, size_t lds_limit, int force_path = 0,
                     int64_t steps_hint = 0) {
    LinearPlan p;
    p.n_tiles16 = 1;
    // more than 16 rows: the wide kernel, except at 17-32 rows on large matrices, where the skinny kernel's pure
    // weight streaming still wins.  4 bit: from 40 MB with rows of 8192 columns and more, 16 wavefronts side by side
    // (6-20 % faster on the 70B and 405B shapes except the 70B o matrix; the wide kernel wins on every 8B shape).
    // 8 bit: above 256 MB, the same 16-wavefront shape (with K split to one round of workgroups it is 15-20 % faster
    // than 8 wavefronts on the 70B gate_up and 405B qkv matrices and level on the 405B gate_up and down matrices).
    const size_t packed_bytes = (size_t)N * K * bits / 8;
    const bool streams16 = M <= 32 && ((bits == 4 && packed_bytes >= ((size_t)40 << 20) && K >= 8192) ||
                                       packed_bytes > ((size_t)256 << 20));
    const bool streams_at_32 = streams16;
    const bool wide_wins = g % 128 == 0 && M > 16 && !streams_at_32;
    // 128 rows and more, and enough 128 x 256 output tiles to fill 9/16 of the compute units without splitting K:
    // the tile kernel (measured against the wide kernel on the 8B, 70B and 405B shapes at M = 128 ... 4096: it wins
    // by 8-15 % from 144 tiles and loses from 128 down), unless its 128-row padding costs more than the wide
    // kernel's 64-row padding
    const bool tile_wins = g % 128 == 0 && M >= 128 && ((N + 255) / 256) * ((M + 127) / 128) >= 144 &&
                           (M + 127) / 128 * 2 <= (M + 63) / 64;
    // Below 144 tiles the tile kernel can still win by splitting K (deep matrices: the wide kernel would split as well
    // and re-reads its activations more often): taken when its modelled time is under 1.075 x the wide plan's (the
    // two models are calibrated apart by about that much).  Measured on the 8B, 70B and 405B shapes at 128-1024
    // rows: 5-27 % faster on the points this picks (8B down from 384 rows, 70B qkv at 256, 70B down from 256, 405B
    // qkv at 128, 405B o and down from 192; 8B gate_up at 320 is 6 % slower).  Where the 128-row wide variant
    // (below) applies under 192 rows it keeps the matrix.  8-bit weights: level on average (+12 % to -9 %), so they
    // keep the 144-tile rule.
    const bool tall_wide = wide_wins && bits == 4 && M >= 128 && (M + 127) / 128 * 2 <= (M + 63) / 64 &&
                           packed_bytes >= ((size_t)40 << 20) && K > N;
    bool tile_by_model = false;
    if (force_path == 0 && !tile_wins && wide_wins && M >= 128 && bits == 4) {
        LinearPlan w;
        wide_plan(M, N, K, bits, &w);
        int r16 = 4, sk = 1;
        const double t_tile = tile_plan_choose(M, N, K, &r16, &sk);
        const double t_wide = wide_model_us(M, N, K, bits, w.m_rows16, w.waves_n, w.n_tiles16, w.split_k);
        tile_by_model = t_tile * 0.93 < t_wide && !(tall_wide && M < 192);
    }
    if (force_path == 4 || (force_path == 0 && (tile_wins || tile_by_model))) {
        p.path = 4;
        p.prefetch = 1; p.waves_n = 8; p.waves_k = 1;
        tile_plan_choose(M, N, K, &p.m_rows16, &p.split_k);
        p.m_blocks = (int)((M + 32 * p.m_rows16 - 1) / (32 * p.m_rows16));
        return p;
    }
    // 128 rows and more, where the tile kernel has not taken over (in practice 128 to 191 rows), on 4-bit matrices of
    // 40 MB and more with more input than output columns (the down projections): the wide kernel's 128-row variant
    // with K split until there is a workgroup per compute unit.  3-12 % faster than the 64-row variant on the 70B and
    // 405B down matrices; within +-7 % on their qkv and o matrices, slower on every 8B shape, and on 8-bit weights
    // ahead on one matrix only, so those keep the 64-row variant.
    if (force_path == 0 && tall_wide) {
        p.path = 3;
        p.prefetch = 1; p.waves_n = 8; p.waves_k = 1; p.n_tiles16 = 2;
        p.m_rows16 = 8;
        p.m_blocks = (int)((M + 127) / 128);
        p.split_k = tall_wide_split(M, N, K);
        return p;
    }
    if (force_path == 3 || (force_path == 0 && wide_wins)) {
        wide_plan(M, N, K, bits, &p);
        return p;
    }
    if (M <= 16 && steps_hint == 0) {
        // the table lookup costs tens of microseconds of host time (logarithms over ~800 entries): remembered per problem
        struct Key { int64_t M, N, K; int bits; size_t lds; };
        struct Memo { Key k; LinearPlan p; bool ok; };
        static std::mutex memo_mutex;
        static std::vector<Memo> memo;
        {
            std::lock_guard<std::mutex> lock(memo_mutex);
            for (const Memo& m : memo)
                if (m.k.M == M && m.k.N == N && m.k.K == K && m.k.bits == bits && m.k.lds == lds_limit) {
                    if (m.ok) return m.p;
                    goto rules;
                }
        }
        {
            const bool ok = skinny_plan_from_table(M, N, K, bits, lds_limit, &p);
            std::lock_guard<std::mutex> lock(memo_mutex);
            if (memo.size() >= 4096) memo.clear();              // a serving process sees a handful of shapes; bound it anyway
            memo.push_back({{M, N, K, bits, lds_limit}, p, ok});
            if (ok) return p;
        }
    }
rules:
    p.n_tiles16 = 1;
    // (no usable table entry, more than 16 rows on this kernel, or a slice of a grouped launch: the rules below)
    const int64_t NT = N / 16, KC = K / chunk_k(bits);
    // 4 KiB chunk-steps in the whole matrix, or in everything that shares the launch (grouped call)
    const int64_t steps = NT * KC > steps_hint ? NT * KC : steps_hint;
    p.m_rows16 = M <= 16 ? 1 : (M <= 32 ? 2 : 4);              // weights are streamed once per 16/32/64 rows
    const int mrows = 16 * p.m_rows16;
    const int rows = (int)(M < mrows ? M + 1 : mrows);
    p.path = 1;
    p.m_blocks = (int)((M + mrows - 1) / mrows);
    p.prefetch = 1;
    p.split_k = 1;
    // Matrices of a hundred megabytes and more with long rows (more than 16 chunks): the launch is many generations of
    // workgroups, its fixed costs no longer count, and what matters is the activation traffic from L2 (M / (4 waves_n)
    // of the weight bytes, whatever the K split) and enough, not too long-lived, workgroups.  From sweeps over
    // (waves_n, waves_k, split_k, prefetch) on the 70B and 405B shapes at 1-16 rows (choice within 10 % of the best
    // measured configuration everywhere, 3 % on average).
    const size_t wbytes = (size_t)N * (size_t)K * (size_t)bits / 8;
    if (KC > 16 && wbytes >= ((size_t)100 << 20) && rows <= 16) {
        if (rows == 2) {                                       // one row: eight wavefronts along K, K in halves up to 32 chunks
            p.waves_n = 1; p.waves_k = 8; p.split_k = KC <= 32 ? 2 : 1;
        } else if (rows == 3 && KC <= 32) {
            p.waves_n = 2; p.waves_k = 2; p.split_k = 4;
        } else {
            // eight tile-rows share the staged rows; K is split across workgroups to fill the compute units
            p.waves_n = 8; p.waves_k = 1; p.split_k = 1;
            // (two of these workgroups share a compute unit: as many splits as keep the launch within one round of 512;
            // three on the 405B qkv matrix, 144 workgroups each, are 9-14 % faster than four)
            int64_t split = 512 / ((NT + 7) / 8);
            split = split < 1 ? 1 : (split > 8 ? 8 : split);
            while (split > 1 && (KC / split < 4 || (size_t)M * N * sizeof(float) * split > kWorkspaceCap)) --split;
            p.split_k = (int)split;
        }
    } else
    // up to 4 rows on a moderately long K (K = 14336: 28 chunks) also stream best unsplit: 14 wavefronts x 2 chunks
    if (rows <= 2 || (rows == 3 && KC >= 16) || (rows <= 5 && KC > 16 && KC <= 32 && NT <= 384)) {
        const int64_t per_wave = steps <= 6144 ? 1 : (steps <= 24576 ? 2 : 4);
        const int64_t even = (KC + per_wave - 1) / per_wave;   // wavefronts that each get exactly per_wave chunks
        if (even <= 16 && KC % even == 0) {
            p.waves_k = (int)even;                             // e.g. K = 14336: 28 chunks = 14 wavefronts x 2
        } else {
            p.waves_k = round_pow2(even, 1, 16);
            while (p.waves_k > KC) p.waves_k /= 2;
        }
        p.waves_n = (steps > 24576 && p.waves_k < 8) ? 8 / p.waves_k : 1;    // eight wavefronts only for the largest
        if (p.waves_k > 8 && KC == 16) {                       // 16 one-chunk wavefronts: two tile-rows of 8 do better (8-bit 8B qkv)
            p.waves_k = 8;
            p.waves_n = NT >= 384 ? 2 : 1;
        }
    } else if (steps <= 6144) {
        p.waves_k = round_pow2(KC, 1, 8);
        while (p.waves_k > KC) p.waves_k /= 2;
        p.waves_n = NT >= 384 ? 2 : 1;
    } else if (rows <= 16) {
        if (KC > 16) {                                         // long K: about 7-14 chunks per workgroup
            p.waves_n = (rows <= 5 && KC <= 32) ? 2 : 4;       // few rows: two tile-rows share them, more workgroups
            p.waves_k = KC <= 32 ? 4 : 2;
            int64_t split = 4;
            while (split > 1 && (size_t)M * N * sizeof(float) * split > kWorkspaceCap) --split;
            p.split_k = (int)split;
        } else if (steps > 24576 && NT <= 2048) {              // many chunk-steps in few tile-rows (8-bit 8B gate_up)
            p.waves_n = 4;
            p.waves_k = 2;
        } else if (steps > 24576) {                            // the largest matrices: long-lived wavefronts
            p.waves_n = rows <= 5 ? 2 : 8;
            p.waves_k = rows <= 5 ? 2 : 1;
        } else if (KC >= 16) {                                 // K = 8192 on matrices of 30-60 MB (sweeps on the 70B qkv and o)
            if (rows <= 5) { p.waves_n = 2; p.waves_k = 4; }
            else if (rows <= 9) { p.waves_n = 4; p.waves_k = 4; p.split_k = 4; }
            else { p.waves_n = 8; p.waves_k = 2; p.split_k = 4; }
            while (p.split_k > 1 && (size_t)M * N * sizeof(float) * p.split_k > kWorkspaceCap) p.split_k /= 2;
        } else {
            p.waves_n = 4;
            p.waves_k = rows <= 9 ? 4 : 2;
        }
    } else {
        // more than 16 rows: wide workgroups share the staged rows (16 wavefronts on the large matrices that stay on
        // this kernel at 17-32 rows); K is split across workgroups only as far as needed to occupy the compute units
        p.waves_n = streams16 ? 16 : 8;
        p.waves_k = 1;
        const int64_t wgs = ((NT + 15) / 16) * p.m_blocks;
        if (streams16) {
            // one 16-wavefront workgroup runs per compute unit: as many splits as keep the launch within one round of
            // 256 (72 workgroups x 3 on the 405B qkv matrix: 45 us against 55 with two splits, 61-65 with four);
            // five to seven splits measured level with four
            int64_t s = 256 / wgs;
            s = s < 1 ? 1 : (s > 8 ? 8 : (s > 4 && s < 8 ? 4 : s));
            while (s > 1 && (s > KC || (size_t)M * N * sizeof(float) * s > kWorkspaceCap)) --s;
            p.split_k = (int)s;
        } else {
            while (wgs * p.split_k < 256 && p.split_k * 2 <= kMaxSplitK && p.split_k * 2 <= KC &&
                   (size_t)M * N * sizeof(float) * (p.split_k * 2) <= kWorkspaceCap)
                p.split_k *= 2;
        }
    }
    while (p.waves_n > 1 && p.waves_n > NT) p.waves_n /= 2;
    LinearArgs a;
    a.M = M; a.N = N; a.K = K; a.bits = bits; a.g = K;
    while (!rtn::linear_plan_fits(a, p, lds_limit) && p.waves_n < 16) {   // more threads to stage the rows
        p.waves_n *= 2;
        while (p.waves_n * p.waves_k > 16) p.waves_k /= 2;
    }
    return p;
}

rtn_status resolve_plan(const LinearArgs& a, const rtn_linear_cfg* cfg, size_t workspace_nbytes, LinearPlan* out) {
    const size_t lds_limit = (size_t)device_max_lds();
    LinearPlan p = auto_plan(a.M, a.N, a.K, a.bits, a.g, lds_limit, cfg ? cfg->path : 0);
    if (cfg) {
        if (cfg->path) p.path = cfg->path;
        if (cfg->prefetch) p.prefetch = cfg->prefetch;
        if (cfg->waves_n) p.waves_n = cfg->waves_n;
        if (cfg->waves_k) p.waves_k = cfg->waves_k;
        if (cfg->split_k) p.split_k = cfg->split_k;
        if (cfg->m_rows16) {
            p.m_rows16 = cfg->m_rows16;
            p.m_blocks = (int)((a.M + 16 * p.m_rows16 - 1) / (16 * p.m_rows16));
        }
        if (cfg->n_tiles16) p.n_tiles16 = cfg->n_tiles16;
        // the vector-ALU variant and several row blocks per wavefront keep one chunk in flight: an automatic plan's deeper
        // prefetch does not carry over to them unless asked for
        if (!cfg->prefetch && (p.path == 2 || (p.path == 1 && p.m_rows16 > 1))) p.prefetch = 1;
        if (p.path == 4 && !cfg->m_rows16 && cfg->split_k) p.m_rows16 = 0;     // a given split: height chosen at launch
    }
    const int64_t KC = a.K / chunk_k(a.bits);
    if (p.path < 1 || p.path > 4) return RTN_ERR_CONFIG;
    // wide and tile kernels: a split the caller did not ask for shrinks to what the workspace passed can hold (slower,
    // not an error; the skinny kernel's plans tie the staged slice to the split, so there it stays an error)
    if (p.path >= 3 && !(cfg && cfg->split_k) && p.split_k > 1) {
        const size_t one = (size_t)a.M * a.N * sizeof(float);
        const size_t fit = a.workspace ? workspace_nbytes / one : 0;
        if ((size_t)p.split_k > fit) p.split_k = fit < 1 ? 1 : (int)fit;
    }
    if (p.path >= 3) {
        const bool ok = p.path == 3 ? rtn::wide_plan_valid(a, p) : rtn::tile_plan_valid(a, p);
        if (!ok || p.split_k > kMaxSplitK) return RTN_ERR_CONFIG;
        if ((uint64_t)a.N * a.K * a.bits / 8 >= 0x7FFF0000ull || (uint64_t)a.M * a.K * 2 >= 0x7FFF0000ull)
            return RTN_ERR_SHAPE;                               // 32-bit buffer offsets
        if (p.split_k > 1) {
            const size_t need = (size_t)a.M * a.N * sizeof(float) * p.split_k;
            if (a.workspace == nullptr || workspace_nbytes < need) return RTN_ERR_WORKSPACE;
        }
        *out = p;
        return RTN_OK;
    }
    if (p.path == 2 && (a.M > 4 || p.prefetch != 1 || p.m_rows16 != 1 || a.g < tile_k(a.bits))) return RTN_ERR_CONFIG;
    if (p.prefetch != 1 && p.prefetch != 2 && p.prefetch != 4) return RTN_ERR_CONFIG;
    if (p.m_rows16 != 1 && p.m_rows16 != 2 && p.m_rows16 != 4) return RTN_ERR_CONFIG;
    if (p.m_rows16 > 1 && p.prefetch != 1) return RTN_ERR_CONFIG;
    if (p.waves_n < 1 || p.waves_k < 1 || p.waves_n * p.waves_k > 16) return RTN_ERR_CONFIG;
    if (p.split_k < 1 || p.split_k > kMaxSplitK || p.split_k > KC) return RTN_ERR_CONFIG;
    if (!rtn::linear_plan_fits(a, p, lds_limit)) return RTN_ERR_CONFIG;
    if ((uint64_t)a.N * a.K * a.bits / 8 >= 0x7FFF0000ull || (uint64_t)a.M * a.K * 2 >= 0x7FFF0000ull)
        return RTN_ERR_SHAPE;                                   // 32-bit buffer offsets
    if (p.split_k > 1) {
        const size_t need = (size_t)a.M * a.N * sizeof(float) * p.split_k;
        if (a.workspace == nullptr || workspace_nbytes < need) return RTN_ERR_WORKSPACE;
    }
    *out = p;
    return RTN_OK;
}

// ---- split-K partial sums for the entry point that allocates nothing ----------------------------------------------
// A fixed device array takes the place of the caller's workspace.  Every GPU the library runs on holds its own copy
// (at its own address) until the process ends.  In host code the array's name is only a handle for the runtime: the
// device address is looked up once per device, with that device current, and kept; kernels and everything else
// only ever see that address.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

rtn_status scratch_for_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RTN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return RTN_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RTN_OK;
}

}  // namespace

extern "C" {

const char* rtn_status_str(rtn_status s) {
    switch (static_cast<int>(s)) {             // callers from C or a foreign-function interface may pass any integer
        case RTN_OK: return "ok";
        case RTN_ERR_NULL: return "null pointer";
        case RTN_ERR_BITS: return "bits must be 4 or 8";
        case RTN_ERR_GROUP: return "unsupported group size";
        case RTN_ERR_SHAPE: return "unsupported shape";
        case RTN_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case RTN_ERR_WORKSPACE: return "workspace too small";
        case RTN_ERR_CONFIG: return "invalid kernel configuration";
        case RTN_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

int rtn_layout_version(void) { return 1; }

size_t rtn_qweight_nbytes(int64_t N, int64_t K, int bits) {
    int64_t g;
    if (check_problem(N, K, bits, 0, &g) != RTN_OK) return 0;
    return (size_t)N * (size_t)K * (size_t)bits / 8;
}

size_t rtn_scales_nbytes(int64_t N, int64_t K, int group_size) {
    if (N <= 0 || K <= 0) return 0;
    int64_t g = group_size <= 0 ? K : group_size;
    if (g > K || K % g != 0) return 0;
    return (size_t)N * (size_t)(K / g) * 2;
}

size_t rtn_workspace_nbytes(int64_t M, int64_t N, int64_t K, int bits, int group_size) {
    int64_t g;
    if (M <= 0 || check_problem(N, K, bits, group_size, &g) != RTN_OK) return 0;
    size_t bound = workspace_bound(M, N);
    const LinearPlan p = auto_plan(M, N, K, bits, g, (size_t)device_max_lds());
    if (p.split_k > 1) {                                        // the automatic plan's own need, where it is larger
        const size_t need = ((size_t)M * (size_t)N * sizeof(float) * (size_t)p.split_k + 255) & ~(size_t)255;
        if (need > bound) bound = need;
    }
    const int64_t rows_first = p.path == 4 ? tile_two_launches(M, N, K) : 0;
    for (int part = 0; rows_first > 0 && part < 2; ++part) {    // and of the two launches rtn_linear would issue
        const int64_t rows = part == 0 ? rows_first : M - rows_first;
        int r16, sk;
        tile_plan_choose(rows, N, K, &r16, &sk);
        const size_t need = sk > 1 ? (((size_t)rows * (size_t)N * sizeof(float) * (size_t)sk + 255) & ~(size_t)255) : 0;
        if (need > bound) bound = need;
    }
    return bound;
}

rtn_status rtn_quantize(const void* dev_W, int64_t N, int64_t K, int bits, int group_size, int flags,
                        void* dev_qweight, void* dev_scales, void* stream) {
    if (!dev_W || !dev_qweight || !dev_scales) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (flags != RTN_SCALE_QMAX && flags != RTN_SCALE_EQ2) return RTN_ERR_CONFIG;
    if (!aligned16(dev_W) || !aligned16(dev_qweight) || !aligned16(dev_scales)) return RTN_ERR_ALIGN;
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const float divisor = (flags == RTN_SCALE_EQ2) ? qmax + 0.5f : qmax;
    hipError_t e = rtn::launch_quantize(dev_W, N, K, bits, g, divisor, dev_qweight, dev_scales,
                                        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_linear_ex(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                         int64_t N, int64_t K, int bits, int group_size, void* dev_C,
                         void* dev_workspace, size_t workspace_nbytes, void* stream,
                         const rtn_linear_cfg* cfg) {
    if (!dev_A || !dev_qweight || !dev_scales || !dev_C) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (M <= 0 || M > (1 << 20)) return RTN_ERR_SHAPE;
    if (!aligned16(dev_A) || !aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_C) ||
        !aligned16(dev_workspace))
        return RTN_ERR_ALIGN;
    LinearArgs a;
    a.A = dev_A; a.qweight = dev_qweight; a.scales = dev_scales; a.C = dev_C;
    a.workspace = static_cast<float*>(dev_workspace);
    a.M = M; a.N = N; a.K = K; a.g = g; a.bits = bits;
    LinearPlan p;
    st = resolve_plan(a, cfg, workspace_nbytes, &p);
    if (st != RTN_OK) return st;
    const int64_t rows_first = (!cfg && p.path == 4) ? tile_two_launches(M, N, K) : 0;
    if (rows_first > 0) {
        rtn_linear_cfg tile_cfg = {};
        tile_cfg.path = 4;
        for (int part = 0; part < 2; ++part) {
            LinearArgs b = a;
            const int64_t r0 = part == 0 ? 0 : rows_first;
            b.M = part == 0 ? rows_first : M - rows_first;
            b.A = static_cast<const char*>(dev_A) + (size_t)r0 * K * 2;
            b.C = static_cast<char*>(dev_C) + (size_t)r0 * N * 2;
            st = resolve_plan(b, &tile_cfg, workspace_nbytes, &p);
            if (st != RTN_OK) return st;
            if (rtn::launch_linear(b, p, static_cast<hipStream_t>(stream)) != hipSuccess) return RTN_ERR_HIP;
        }
        return RTN_OK;
    }
    hipError_t e = rtn::launch_linear(a, p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_linear(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                      int64_t N, int64_t K, int bits, int group_size, void* dev_C,
                      void* dev_workspace, size_t workspace_nbytes, void* stream) {
    return rtn_linear_ex(dev_A, M, dev_qweight, dev_scales, N, K, bits, group_size, dev_C, dev_workspace,
                         workspace_nbytes, stream, nullptr);
}

rtn_status rtn_problem_status(int64_t N, int64_t K, int bits, int group_size) {
    int64_t g;
    return check_problem(N, K, bits, group_size, &g);
}

rtn_status rtn_linear_validate(int64_t M, int64_t N, int64_t K, int bits, int group_size, size_t workspace_nbytes,
                               const rtn_linear_cfg* cfg) {
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (M <= 0 || M > (1 << 20)) return RTN_ERR_SHAPE;
    LinearArgs a;
    a.A = nullptr; a.qweight = nullptr; a.scales = nullptr; a.C = nullptr;
    // only "is there a workspace" matters to the plan checks; nothing is launched and the address is never used
    static float workspace_stand_in;
    a.workspace = workspace_nbytes > 0 ? &workspace_stand_in : nullptr;
    a.M = M; a.N = N; a.K = K; a.g = g; a.bits = bits;
    LinearPlan p;
    return resolve_plan(a, cfg, workspace_nbytes, &p);
}

rtn_status rtn_linear_noalloc(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                              int64_t N, int64_t K, int bits, int group_size, void* dev_C, void* stream) {
    if (!dev_A || !dev_qweight || !dev_scales || !dev_C) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (M <= 0 || M > (1 << 20)) return RTN_ERR_SHAPE;
    if (rtn_workspace_nbytes(M, N, K, bits, group_size) > kScratchBytes) return RTN_ERR_WORKSPACE;
    void* ptr = nullptr;
    st = scratch_for_current_device(&ptr);
    if (st != RTN_OK) return st;
    return rtn_linear_ex(dev_A, M, dev_qweight, dev_scales, N, K, bits, group_size, dev_C, ptr, kScratchBytes, stream,
                         nullptr);
}

rtn_status rtn_linear_query(int64_t M, int64_t N, int64_t K, int bits, int group_size, rtn_linear_cfg* out) {
    if (!out) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (M <= 0 || M > (1 << 20)) return RTN_ERR_SHAPE;
    if ((uint64_t)N * K * bits / 8 >= 0x7FFF0000ull || (uint64_t)M * K * 2 >= 0x7FFF0000ull)
        return RTN_ERR_SHAPE;                                   // what rtn_linear refuses (32-bit buffer offsets)
    LinearPlan p = auto_plan(M, N, K, bits, g, (size_t)device_max_lds());
    out->path = p.path; out->prefetch = p.prefetch; out->waves_n = p.waves_n;
    out->waves_k = p.waves_k; out->split_k = p.split_k; out->m_rows16 = p.m_rows16;
    out->n_tiles16 = p.n_tiles16;
    return RTN_OK;
}

rtn_status rtn_unpack(const void* dev_qweight, int64_t N, int64_t K, int bits, void* dev_codes_i8, void* stream) {
    if (!dev_qweight || !dev_codes_i8) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, 0, &g);
    if (st != RTN_OK) return st;
    if (!aligned16(dev_qweight) || !aligned16(dev_codes_i8)) return RTN_ERR_ALIGN;
    hipError_t e = rtn::launch_unpack(dev_qweight, nullptr, N, K, bits, K, false, dev_codes_i8,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_dequantize(const void* dev_qweight, const void* dev_scales, int64_t N, int64_t K, int bits,
                          int group_size, void* dev_W_fp16, void* stream) {
    if (!dev_qweight || !dev_scales || !dev_W_fp16) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (!aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_W_fp16)) return RTN_ERR_ALIGN;
    hipError_t e = rtn::launch_unpack(dev_qweight, dev_scales, N, K, bits, g, true, dev_W_fp16,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

size_t rtn_quantize_host_staging_nbytes(int64_t K, int64_t rows_per_shard) {
    if (K <= 0 || rows_per_shard <= 0 || rows_per_shard % 16 != 0) return 0;
    return 2 * (size_t)rows_per_shard * (size_t)K * 2;
}

rtn_status rtn_quantize_from_host(const void* host_W, int64_t N, int64_t K, int bits, int group_size, int flags,
                                  void* dev_qweight, void* dev_scales, void* dev_staging, size_t staging_nbytes,
                                  int64_t rows_per_shard, void* stream, void* copy_stream) {
    if (!host_W || !dev_qweight || !dev_scales || !dev_staging) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (flags != RTN_SCALE_QMAX && flags != RTN_SCALE_EQ2) return RTN_ERR_CONFIG;
    if (rows_per_shard <= 0 || rows_per_shard % 16 != 0) return RTN_ERR_SHAPE;
    if (!aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_staging)) return RTN_ERR_ALIGN;
    if (staging_nbytes < rtn_quantize_host_staging_nbytes(K, rows_per_shard)) return RTN_ERR_WORKSPACE;
    if (stream == copy_stream) return RTN_ERR_CONFIG;          // the overlap needs two streams
    hipStream_t qs = static_cast<hipStream_t>(stream), cs = static_cast<hipStream_t>(copy_stream);
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const float divisor = (flags == RTN_SCALE_EQ2) ? qmax + 0.5f : qmax;
    const size_t shard_bytes = (size_t)rows_per_shard * K * 2;
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};   // start, copied[0..1], consumed[0..1]
    bool ok = true;
    for (int i = 0; i < 5 && ok; ++i) ok = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) {                                                  // destroy what was created before the failure
        for (int i = 0; i < 5; ++i)
            if (ev[i]) (void)hipEventDestroy(ev[i]);
        return RTN_ERR_HIP;
    }
    hipEvent_t start = ev[0], *copied = &ev[1], *consumed = &ev[3];
    // the copy stream starts after whatever the caller queued on `stream` before this call (the staging buffer
    // may still be in use there)
    ok = hipEventRecord(start, qs) == hipSuccess && hipStreamWaitEvent(cs, start, 0) == hipSuccess;
    int64_t shard = 0;
    for (int64_t r0 = 0; r0 < N && ok; r0 += rows_per_shard, ++shard) {
        const int b = (int)(shard & 1);
        const int64_t rows = (N - r0 < rows_per_shard) ? N - r0 : rows_per_shard;
        uint8_t* stage = static_cast<uint8_t*>(dev_staging) + (size_t)b * shard_bytes;
        // copy shard -> staging buffer b, once the quantise pass that last read buffer b is done
        if (shard >= 2) ok = ok && hipStreamWaitEvent(cs, consumed[b], 0) == hipSuccess;
        ok = ok && hipMemcpyAsync(stage, static_cast<const uint8_t*>(host_W) + (size_t)r0 * K * 2, (size_t)rows * K * 2,
                                  hipMemcpyHostToDevice, cs) == hipSuccess;
        ok = ok && hipEventRecord(copied[b], cs) == hipSuccess;
        // quantise it on `stream` into its slice of the packed tensor (tile-rows and scale rows are contiguous)
        ok = ok && hipStreamWaitEvent(qs, copied[b], 0) == hipSuccess;
        if (ok) {
            uint8_t* qdst = static_cast<uint8_t*>(dev_qweight) + (size_t)r0 * K * bits / 8;
            uint8_t* sdst = static_cast<uint8_t*>(dev_scales) + (size_t)r0 * (K / g) * 2;
            ok = rtn::launch_quantize(stage, rows, K, bits, g, divisor, qdst, sdst, qs) == hipSuccess;
        }
        ok = ok && hipEventRecord(consumed[b], qs) == hipSuccess;
    }
    (void)hipEventDestroy(start);
    for (int i = 0; i < 2; ++i) {
        (void)hipEventDestroy(copied[i]);                       // destruction is deferred until the events complete
        (void)hipEventDestroy(consumed[i]);
    }
    return ok ? RTN_OK : RTN_ERR_HIP;
}

// K split of the dense GEMM: the candidate (1-8 splits, not only powers of two) with the lowest modelled time, as for
// the fused tile kernel.  A 128 x 256 tile advances one 64-column step per ~1 us whether or not all compute units
// have a tile (measured: 59-62 us at K = 4096 for 24 to 192 tiles), a 256-row tile takes 1.7 times as long (the
// launch picks the height from the rounds of 256 workgroups each would take); a workgroup costs 8 us besides, and a
// split adds the partials' round trip through the workspace (write and read of split x M x N fp32 at ~4.5 TB/s) and
// the reduce launch.
static int dense_split(int64_t M, int64_t N, int64_t K, size_t workspace_nbytes, double* time_us = nullptr) {
    const int64_t xb = (N + 255) / 256;
    int best = 1;
    double best_t = 1e30;
    for (int s = 1; s <= 8; ++s) {
        if (s > 1 && (K / 128 / s < 8 || (size_t)M * N * sizeof(float) * s > workspace_nbytes)) break;
        const double r_short = (double)((xb * ((M + 127) / 128) * s + 255) / 256);
        const double r_tall = (double)((xb * ((M + 255) / 256) * s + 255) / 256);
        const bool tall = M > 128 && 1.7 * r_tall < r_short;
        const double steps = (double)((K / 64 + s - 1) / s);
        double t = tall ? r_tall * (steps * 1.7 + 8.0) : r_short * (steps * 1.0 + 8.0);
        if (s > 1) t += 2.5 + (2.0 * s * M * N * 4.0 + 2.0 * M * N) / 4.5e6;
        if (t < best_t) {
            best_t = t;
            best = s;
        }
    }
    if (time_us) *time_us = best_t;
    return best;
}

// The dense GEMM in two launches, as rtn_linear does with the fused tile kernel: the first rows (a multiple of 256) as
// full rounds, the rest with the K split that fills its round; 0 where one launch is modelled within 7 % of that.
static int64_t dense_two_launches(int64_t M, int64_t N, int64_t K, size_t workspace_nbytes) {
    if (M > 16384) return 0;                                   // many rounds: the last one no longer matters
    double single = 0, t1 = 0, t2 = 0;
    dense_split(M, N, K, workspace_nbytes, &single);
    double best = single * 0.93;
    int64_t rows_first = 0;
    for (int64_t r1 = 256; r1 < M; r1 += 256) {
        dense_split(r1, N, K, workspace_nbytes, &t1);
        dense_split(M - r1, N, K, workspace_nbytes, &t2);
        if (t1 + t2 < best) { best = t1 + t2; rows_first = r1; }
    }
    return rows_first;
}

rtn_status rtn_gemm_fp16(const void* dev_A, int64_t M, const void* dev_W_fp16, int64_t N, int64_t K, void* dev_C,
                         void* dev_workspace, size_t workspace_nbytes, void* stream) {
    if (!dev_A || !dev_W_fp16 || !dev_C) return RTN_ERR_NULL;
    if (M <= 0 || M > (1 << 20) || N <= 0 || N % 16 != 0 || K <= 0 || K % 128 != 0) return RTN_ERR_SHAPE;
    if ((uint64_t)K * 2 * 128 >= 0x7FFF0000ull) return RTN_ERR_SHAPE;          // one 128-row slab per buffer resource
    if (!aligned16(dev_A) || !aligned16(dev_W_fp16) || !aligned16(dev_C) || !aligned16(dev_workspace)) return RTN_ERR_ALIGN;
    const int64_t rows_first = dev_workspace ? dense_two_launches(M, N, K, workspace_nbytes) : 0;
    for (int part = 0; rows_first > 0 && part < 2; ++part) {
        const int64_t r0 = part == 0 ? 0 : rows_first, rows = part == 0 ? rows_first : M - rows_first;
        const int s = dense_split(rows, N, K, workspace_nbytes);
        if (rtn::launch_gemm_fp16(static_cast<const char*>(dev_A) + (size_t)r0 * K * 2, dev_W_fp16,
                                  static_cast<char*>(dev_C) + (size_t)r0 * N * 2, static_cast<float*>(dev_workspace),
                                  rows, N, K, s, static_cast<hipStream_t>(stream)) != hipSuccess)
            return RTN_ERR_HIP;
    }
    if (rows_first > 0) return RTN_OK;
    const int split = dev_workspace ? dense_split(M, N, K, workspace_nbytes) : 1;
    hipError_t e = rtn::launch_gemm_fp16(dev_A, dev_W_fp16, dev_C, static_cast<float*>(dev_workspace), M, N, K, split,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

size_t rtn_dense_weight_nbytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0) return 0;
    return (size_t)N * (size_t)K * 2;
}

rtn_status rtn_linear_dense(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                            int64_t N, int64_t K, int bits, int group_size, void* dev_C, void* dev_W_tmp,
                            size_t w_tmp_nbytes, void* dev_workspace, size_t workspace_nbytes, void* stream) {
    if (!dev_W_tmp) return RTN_ERR_NULL;
    if (w_tmp_nbytes < rtn_dense_weight_nbytes(N, K)) return RTN_ERR_WORKSPACE;
    rtn_status st = rtn_dequantize(dev_qweight, dev_scales, N, K, bits, group_size, dev_W_tmp, stream);
    if (st != RTN_OK) return st;
    return rtn_gemm_fp16(dev_A, M, dev_W_tmp, N, K, dev_C, dev_workspace, workspace_nbytes, stream);
}

rtn_status rtn_layer_forward(const rtn_module* mods, int n_mods, void* dev_workspace, size_t workspace_nbytes,
                             void* stream) {
    if (!mods) return RTN_ERR_NULL;
    if (n_mods <= 0) return RTN_ERR_SHAPE;
    for (int i = 0; i < n_mods; ++i) {
        const rtn_module& m = mods[i];
        rtn_status st = rtn_linear(m.dev_A, m.M, m.dev_qweight, m.dev_scales, m.N, m.K, m.bits, m.group_size,
                                   m.dev_C, dev_workspace, workspace_nbytes, stream);
        if (st != RTN_OK) return st;
    }
    return RTN_OK;
}

rtn_status rtn_quantize_asym(const void* dev_W, int64_t N, int64_t K, int bits, int group_size,
                             void* dev_qweight, void* dev_scales, void* dev_zeros, void* stream) {
    if (!dev_W || !dev_qweight || !dev_scales || !dev_zeros) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (!aligned16(dev_W) || !aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_zeros))
        return RTN_ERR_ALIGN;
    hipError_t e = rtn::launch_quantize_asym(dev_W, N, K, bits, g, dev_qweight, dev_scales, dev_zeros,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_dequantize_asym(const void* dev_qweight, const void* dev_scales, const void* dev_zeros,
                               int64_t N, int64_t K, int bits, int group_size, void* dev_W_fp16, void* stream) {
    if (!dev_qweight || !dev_scales || !dev_zeros || !dev_W_fp16) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (!aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_zeros) || !aligned16(dev_W_fp16))
        return RTN_ERR_ALIGN;
    hipError_t e = rtn::launch_unpack(dev_qweight, dev_scales, N, K, bits, g, true, dev_W_fp16,
                                      static_cast<hipStream_t>(stream), dev_zeros);
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_linear_asym(const void* dev_A, int64_t M, const void* dev_qweight, const void* dev_scales,
                           const void* dev_zeros, int64_t N, int64_t K, int bits, int group_size,
                           void* dev_C, void* dev_workspace, size_t workspace_nbytes, void* stream) {
    if (!dev_A || !dev_qweight || !dev_scales || !dev_zeros || !dev_C) return RTN_ERR_NULL;
    int64_t g;
    rtn_status st = check_problem(N, K, bits, group_size, &g);
    if (st != RTN_OK) return st;
    if (M <= 0 || M > (1 << 20)) return RTN_ERR_SHAPE;
    if (!aligned16(dev_A) || !aligned16(dev_qweight) || !aligned16(dev_scales) || !aligned16(dev_zeros) ||
        !aligned16(dev_C) || !aligned16(dev_workspace))
        return RTN_ERR_ALIGN;
    LinearArgs a;
    a.A = dev_A; a.qweight = dev_qweight; a.scales = dev_scales; a.C = dev_C; a.zeros = dev_zeros;
    a.workspace = static_cast<float*>(dev_workspace);
    a.M = M; a.N = N; a.K = K; a.g = g; a.bits = bits;
    LinearPlan p;
    rtn_linear_cfg cfg;
    bool planned = false;
    if (M > 16 && g % 128 == 0) {
        // the wide kernel's zero-point instantiations: 8 wavefronts, at most two tile-rows per wavefront
        LinearPlan h;
        wide_plan(M, N, K, bits, &h);
        cfg.path = 3; cfg.prefetch = 1; cfg.waves_n = 8; cfg.waves_k = 1; cfg.split_k = h.split_k;
        // as many of the plan's K splits as the workspace passed can hold
        const size_t fit = dev_workspace ? workspace_nbytes / ((size_t)M * N * sizeof(float)) : 0;
        if ((size_t)cfg.split_k > fit) cfg.split_k = fit < 1 ? 1 : (int)fit;
        cfg.m_rows16 = h.m_rows16; cfg.n_tiles16 = h.n_tiles16 > 2 ? 2 : h.n_tiles16;
        planned = resolve_plan(a, &cfg, workspace_nbytes, &p) == RTN_OK;
    }
    if (!planned) {
        // the small-batch kernel, 16 rows per workgroup, planned as for min(M, 16) rows
        LinearPlan h = auto_plan(M < 16 ? M : 16, N, K, bits, g, (size_t)device_max_lds(), 1);
        cfg.path = 1; cfg.prefetch = 1; cfg.waves_n = h.waves_n; cfg.waves_k = h.waves_k;
        cfg.split_k = M <= 16 ? h.split_k : 1; cfg.m_rows16 = 1; cfg.n_tiles16 = 1;
        st = resolve_plan(a, &cfg, workspace_nbytes, &p);
        if (st != RTN_OK) return st;
    }
    hipError_t e = rtn::launch_linear(a, p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

rtn_status rtn_grouped_forward(const rtn_module* mods, int n_mods, void* dev_workspace, size_t workspace_nbytes,
                               void* stream) {
    if (!mods) return RTN_ERR_NULL;
    if (n_mods <= 0) return RTN_ERR_SHAPE;
    if (!aligned16(dev_workspace)) return RTN_ERR_ALIGN;
    const size_t lds_limit = (size_t)device_max_lds();
    std::vector<LinearArgs> args((size_t)n_mods);
    std::vector<LinearPlan> plans((size_t)n_mods);
    int64_t steps_total = 0;                                   // of the modules the skinny kernel will serve
    for (int i = 0; i < n_mods; ++i) {
        const rtn_module& m = mods[i];
        if (!m.dev_A || !m.dev_qweight || !m.dev_scales || !m.dev_C) return RTN_ERR_NULL;
        int64_t g;
        rtn_status st = check_problem(m.N, m.K, m.bits, m.group_size, &g);
        if (st != RTN_OK) return st;
        if (m.M <= 0 || m.M > (1 << 20)) return RTN_ERR_SHAPE;
        if (!aligned16(m.dev_A) || !aligned16(m.dev_qweight) || !aligned16(m.dev_scales) || !aligned16(m.dev_C))
            return RTN_ERR_ALIGN;
        LinearArgs& a = args[i];
        a.A = m.dev_A; a.qweight = m.dev_qweight; a.scales = m.dev_scales; a.C = m.dev_C;
        a.workspace = static_cast<float*>(dev_workspace);
        a.M = m.M; a.N = m.N; a.K = m.K; a.g = g; a.bits = m.bits;
        if (m.M <= 16) steps_total += (m.N / 16) * (m.K / chunk_k(m.bits));
    }
    for (int i = 0; i < n_mods; ++i) {
        const LinearArgs& a = args[i];
        // planned as one slice of a launch that streams all the small-batch modules together
        const LinearPlan h = auto_plan(a.M, a.N, a.K, a.bits, a.g, lds_limit, 0, a.M <= 16 ? steps_total : 0);
        rtn_linear_cfg cfg;
        cfg.path = h.path; cfg.prefetch = h.prefetch; cfg.waves_n = h.waves_n; cfg.waves_k = h.waves_k;
        cfg.split_k = h.split_k; cfg.m_rows16 = h.m_rows16; cfg.n_tiles16 = h.n_tiles16;
        rtn_status st = resolve_plan(a, &cfg, workspace_nbytes, &plans[i]);
        if (st == RTN_ERR_CONFIG) st = resolve_plan(a, nullptr, workspace_nbytes, &plans[i]);   // the module's own plan
        if (st != RTN_OK) return st;
    }
    hipError_t e = rtn::launch_linear_grouped(args.data(), plans.data(), n_mods, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RTN_OK : RTN_ERR_HIP;
}

static int layer_selected(int layer, int n_layers, int policy, int X) {
    int start;
    switch (policy) {
        case RTN_POLICY_FIRST: start = 0; break;
        case RTN_POLICY_LAST: start = n_layers - X; break;
        case RTN_POLICY_MIDDLE: start = (n_layers - X) / 2; break;
        default: return -1;
    }
    return (layer >= start && layer < start + X) ? 1 : 0;
}

int rtn_plan_bits(int layer, int n_layers, int module_id, int policy, int X, unsigned module_mask) {
    if (n_layers <= 0 || layer < 0 || layer >= n_layers || X < 0 || X > n_layers) return -1;
    if (module_id < 1 || module_id > 4 || module_mask > 15u) return -1;
    const int sel = layer_selected(layer, n_layers, policy, X);
    if (sel < 0) return -1;
    return (sel && (module_mask >> (module_id - 1) & 1u)) ? 8 : 4;
}

double rtn_plan_effective_bits(int n_layers, const int64_t module_params[4], int policy, int X,
                               unsigned module_mask) {
    if (!module_params || n_layers <= 0) return -1.0;
    long double total = 0, bits = 0;
    for (int l = 0; l < n_layers; ++l)
        for (int m = 1; m <= 4; ++m) {
            const int b = rtn_plan_bits(l, n_layers, m, policy, X, module_mask);
            if (b < 0 || module_params[m - 1] < 0) return -1.0;
            total += (long double)module_params[m - 1];
            bits += (long double)module_params[m - 1] * b;
        }
    return total > 0 ? (double)(bits / total) : -1.0;
}

}  // extern "C"
