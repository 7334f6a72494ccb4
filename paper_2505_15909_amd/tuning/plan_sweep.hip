// Plan-sweep tool of the fused dequantise-GEMM: times rtn_linear_ex under HIP-graph replay, launches rotating over >= 600 MB
// of packed weight copies (random bytes as weights: timing only, nothing is checked), for the automatic plan and for
// explicit (wavefronts along N, along K, K splits, chunks in flight) configurations.  The library is loaded with dlopen.
//   build:  hipcc -O2 -std=c++17 --offload-arch=gfx950 -o plan_sweep plan_sweep.hip -ldl
//   auto :  plan_sweep LIB[,LIB...] {8b|70b|405b|small|@shapes.txt} M1,M2,... [bits] auto
//   sweep:  plan_sweep LIB @shapes.txt M1,M2,... bits sweep WN,WK,SPLIT,PREFETCH ...
// shapes.txt: one "name K N" per line.  The sweep output feeds make_plan_table.py, which writes the table the library's
// plan selection looks up (csrc/skinny_plan_table.inc).
#include <hip/hip_runtime.h>
#include <dlfcn.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <string>
#include <vector>
#include <algorithm>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); fflush(stdout); exit(1);} }while(0)
struct cfg_t { int path, prefetch, waves_n, waves_k, split_k, m_rows16, n_tiles16; };
typedef int (*linear_ex_t)(const void*, int64_t, const void*, const void*, int64_t, int64_t, int, int, void*, void*, size_t, void*, const cfg_t*);
typedef int (*query_t)(int64_t, int64_t, int64_t, int, int, cfg_t*);
struct Lib { std::string name; linear_ex_t lin; query_t query; };
struct Shape { const char* name; int K, N; };
static hipStream_t st;
static hipEvent_t e0, e1;

template <typename F> static double time_graph(F issue, int n_per) {
  hipGraph_t g; hipGraphExec_t ge;
  CK(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));
  issue();
  CK(hipStreamEndCapture(st, &g)); CK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
  CK(hipGraphLaunch(ge, st)); CK(hipStreamSynchronize(st));
  std::vector<double> ts;
  for (int r = 0; r < 7; ++r) {
    CK(hipEventRecord(e0, st)); CK(hipGraphLaunch(ge, st)); CK(hipEventRecord(e1, st)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ts.push_back(ms * 1e3 / n_per);
  }
  CK(hipGraphExecDestroy(ge)); CK(hipGraphDestroy(g));
  std::sort(ts.begin(), ts.end());
  return ts[ts.size() / 2];
}

int main(int argc, char** argv) {
  if (argc < 4) { printf("usage\n"); return 1; }
  std::vector<Lib> libs;
  { char* s = strdup(argv[1]); for (char* t = strtok(s, ","); t; t = strtok(nullptr, ",")) {
      void* h = dlopen(t, RTLD_NOW | RTLD_LOCAL); if (!h) { printf("dlopen %s: %s\n", t, dlerror()); return 1; }
      Lib l; l.name = t; l.lin = (linear_ex_t)dlsym(h, "rtn_linear_ex"); l.query = (query_t)dlsym(h, "rtn_linear_query"); libs.push_back(l); } }
  std::string fam = argv[2];
  std::vector<int> Ms; { char* s = strdup(argv[3]); for (char* t = strtok(s, ","); t; t = strtok(nullptr, ",")) Ms.push_back(atoi(t)); }
  const int bits = argc > 4 ? atoi(argv[4]) : 4;
  const std::string mode = argc > 5 ? argv[5] : "auto";
  const int g = bits == 4 ? 128 : 0;
  std::vector<Shape> shapes;
  if (fam == "8b") shapes = {{"qkv", 4096, 6144}, {"o", 4096, 4096}, {"gate_up", 4096, 28672}, {"down", 14336, 4096}};
  else if (fam == "70b") shapes = {{"qkv", 8192, 10240}, {"o", 8192, 8192}, {"gate_up", 8192, 57344}, {"down", 28672, 8192}};
  else if (fam == "405b") shapes = {{"qkv", 16384, 18432}, {"o", 16384, 16384}, {"gate_up", 16384, 106496}, {"down", 53248, 16384}};
  else if (fam == "small") shapes = {{"l1b_qkv", 2048, 3072}, {"l1b_o", 2048, 2048}, {"l1b_gu", 2048, 16384}, {"l1b_down", 8192, 2048},
                                     {"l3b_qkv", 3072, 5120}, {"l3b_o", 3072, 3072}, {"l3b_gu", 3072, 16384}, {"l3b_down", 8192, 3072}};
  static std::vector<std::string> names;
  if (fam[0] == '@') {            // shapes from a file: name K N per line
    // "@path" or "@path:first:count" (a slice of the file's lines, for runs under a time limit)
    std::string path = fam.substr(1); long first = 0, count = 1 << 30;
    const size_t c1 = path.find(':');
    if (c1 != std::string::npos) { sscanf(path.c_str() + c1 + 1, "%ld:%ld", &first, &count); path = path.substr(0, c1); }
    FILE* f = fopen(path.c_str(), "r"); char nm[64]; int k, n;
    std::vector<std::pair<int, int>> kn;
    for (long i = 0; f && fscanf(f, "%63s %d %d", nm, &k, &n) == 3; ++i)
      if (i >= first && i < first + count) { names.push_back(nm); kn.push_back({k, n}); }
    if (f) fclose(f);
    for (size_t i = 0; i < names.size(); ++i) shapes.push_back({names[i].c_str(), kn[i].first, kn[i].second});
  }
  CK(hipStreamCreate(&st)); CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  size_t max_w = 0; for (auto& sh : shapes) max_w = std::max(max_w, (size_t)sh.N * sh.K * bits / 8);
  const size_t pool_bytes = std::max((size_t)1 << 30, std::min((size_t)3 << 30, 2 * max_w + (1 << 20)));
  uint8_t* pool; CK(hipMalloc(&pool, pool_bytes));
  { std::vector<uint32_t> h(1 << 20); uint32_t x = 12345; for (auto& v : h) { x = x * 1664525u + 1013904223u; v = x; }
    for (size_t o = 0; o < pool_bytes; o += h.size() * 4) CK(hipMemcpy(pool + o, h.data(), std::min(h.size() * 4, pool_bytes - o), hipMemcpyHostToDevice)); }
  const size_t ws_bytes = (size_t)256 << 20;
  void* ws; CK(hipMalloc(&ws, ws_bytes)); CK(hipMemset(ws, 0, ws_bytes));
  int maxM = *std::max_element(Ms.begin(), Ms.end());
  size_t maxK = 0, maxN = 0; for (auto& s : shapes) { maxK = std::max(maxK, (size_t)s.K); maxN = std::max(maxN, (size_t)s.N); }
  _Float16 *A, *C, *S;
  CK(hipMalloc(&A, (size_t)maxM * maxK * 2)); CK(hipMalloc(&C, (size_t)maxM * maxN * 2));
  { std::vector<_Float16> h((size_t)maxM * maxK); uint32_t x = 777; for (auto& v : h) { x = x * 1664525u + 1013904223u; v = (_Float16)(((int)(x >> 16) % 2001 - 1000) * 0.002f); }
    CK(hipMemcpy(A, h.data(), h.size() * 2, hipMemcpyHostToDevice)); }
  size_t maxS = 0; for (auto& s : shapes) maxS = std::max(maxS, (size_t)s.N * (g ? s.K / g : 1));
  CK(hipMalloc(&S, maxS * 2));
  { std::vector<_Float16> h(maxS, (_Float16)0.01f); CK(hipMemcpy(S, h.data(), maxS * 2, hipMemcpyHostToDevice)); }

  auto copies_of = [&](const Shape& s, size_t& bytes) { bytes = (size_t)s.N * s.K * bits / 8; size_t c = std::max<size_t>(2, (600000000 + bytes - 1) / bytes); return (int)std::min(c, pool_bytes / bytes); };

  if (mode == "auto") {
    for (auto& L : libs) {
      printf("## %s  %s int%d\n", L.name.c_str(), fam.c_str(), bits);
      std::vector<double> tot(Ms.size(), 0.0); double totb = 0;
      for (auto& s : shapes) {
        size_t bytes; const int nc = copies_of(s, bytes); const double nb = bytes + (double)s.N * (g ? s.K / g : 1) * 2; totb += nb;
        for (size_t mi = 0; mi < Ms.size(); ++mi) {
          const int M = Ms[mi]; cfg_t q; L.query(M, s.N, s.K, bits, g, &q);
          int bad = 0;
          auto issue = [&]() { for (int r = 0; r < 3; ++r) for (int c = 0; c < nc; ++c) { int rc = L.lin(A, M, pool + (size_t)c * bytes, S, s.N, s.K, bits, g, C, ws, ws_bytes, st, nullptr); if (rc) bad = rc; } };
          issue(); CK(hipStreamSynchronize(st));
          const double t = time_graph(issue, 3 * nc);
          tot[mi] += t;
          printf("%-8s %6d->%6d M=%3d %8.2f us %6.0f GB/s %5.1f %%  path %d %dx%d split %d nb %d rows16 %d%s\n", s.name, s.K, s.N, M, t, nb / t / 1e3, nb / t / 80e3,
                 q.path, q.waves_n, q.waves_k, q.split_k, q.prefetch, q.m_rows16, bad ? "  (ERROR)" : ""); fflush(stdout);
        }
      }
      double step = 0;
      for (size_t mi = 0; mi < Ms.size(); ++mi) { printf("layer set M=%3d: %8.2f us %6.0f GB/s %5.1f %%\n", Ms[mi], tot[mi], totb / tot[mi] / 1e3, totb / tot[mi] / 80e3); step += tot[mi]; }
      printf("sum over M: %.2f us -> %.0f GB/s %.1f %%\n", step, totb * Ms.size() / step / 1e3, totb * Ms.size() / step / 80e3);
      // bench-like step: for each M the four modules back to back, rotating layer copies
      {
        size_t layer_bytes = 0; for (auto& s : shapes) layer_bytes += (size_t)s.N * s.K * bits / 8;
        const int nc = (int)std::min<size_t>(std::max<size_t>(2, (size_t)(2.4 * 256e6 / layer_bytes) + 1), pool_bytes / layer_bytes);
        auto issue = [&]() { int pass = 0; for (int c = 0; c < nc; ++c) for (int M : Ms) { size_t off = (size_t)(pass++ % nc) * layer_bytes;
              for (auto& s : shapes) { L.lin(A, M, pool + off, S, s.N, s.K, bits, g, C, ws, ws_bytes, st, nullptr); off += (size_t)s.N * s.K * bits / 8; } } };
        issue(); CK(hipStreamSynchronize(st));
        const double t = time_graph(issue, nc);
        printf("bench-like step (%d copies): %.2f us per step -> %.0f GB/s %.1f %%\n", nc, t, totb * Ms.size() / t / 1e3, totb * Ms.size() / t / 80e3);
      }
      fflush(stdout);
    }
  } else {   // sweep: explicit plans given as extra args "wn,wk,split,nb[,path]" ...
    std::vector<cfg_t> cfgs;
    for (int i = 6; i < argc; ++i) { cfg_t c = {1, 1, 1, 1, 1, 1, 1}; int path = 1; sscanf(argv[i], "%d,%d,%d,%d,%d", &c.waves_n, &c.waves_k, &c.split_k, &c.prefetch, &path); c.path = path; cfgs.push_back(c); }
    for (auto& L : libs) {
      printf("## sweep %s %s int%d\n", L.name.c_str(), fam.c_str(), bits);
      for (auto& s : shapes) {
        size_t bytes; const int nc = copies_of(s, bytes); const double nb = bytes + (double)s.N * (g ? s.K / g : 1) * 2;
        for (int M : Ms) {
          cfg_t q; L.query(M, s.N, s.K, bits, g, &q);
          std::vector<cfg_t> all = cfgs; all.insert(all.begin(), q);
          for (size_t ci = 0; ci < all.size(); ++ci) {
            cfg_t c = all[ci]; if (ci > 0) { c.m_rows16 = 1; c.n_tiles16 = 1; }
            int rc = L.lin(A, M, pool, S, s.N, s.K, bits, g, C, ws, ws_bytes, st, &c);
            if (rc) { continue; }
            auto issue = [&]() { for (int r = 0; r < 3; ++r) for (int cc = 0; cc < nc; ++cc) L.lin(A, M, pool + (size_t)cc * bytes, S, s.N, s.K, bits, g, C, ws, ws_bytes, st, &c); };
            issue(); CK(hipStreamSynchronize(st));
            const double t = time_graph(issue, 3 * nc);
            printf("%-8s M=%3d %s %2dx%-2d split %2d nb %d : %8.2f us %5.1f %%\n", s.name, M, ci == 0 ? "AUTO" : "    ", c.waves_n, c.waves_k, c.split_k, c.prefetch, t, nb / t / 80e3); fflush(stdout);
          }
        }
      }
    }
  }
  return 0;
}
