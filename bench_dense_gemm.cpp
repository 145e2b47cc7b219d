// Dense fp16 GEMM baseline for bench.py: Y[T x out] = X[T x in] . W[out x in]^T through hipBLASLt
// (fp16 operands, fp32 compute, fp16 result), with the algorithm chosen by measurement: every
// candidate hipblasLtMatmulAlgoGetHeuristic returns (and, with --all, every algorithm of the library
// that supports the problem) is timed on the device and the fastest is kept per shape.
//
// A stand-alone program rather than a module of the Python process: PyTorch ships a hipBLASLt of its
// own under the same soname, and the baseline should be the ROCm installation's library with its own
// search, not whatever the framework's dispatcher picks.
//
// Usage: bench_dense_gemm [--iters N] [--warmup W] [--candidates C] [--all] name:T:out:in ...
// Output: one JSON object on stdout.  "layers" lists, in the order given, the time of each GEMM
// measured the way bench.py measures the sparse product: all layers enqueued in turn, pass after
// pass, HIP events around every GEMM, every layer with operands of its own, so that a GEMM finds its
// weight in HBM and not in the last-level cache.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hipblaslt/hipblaslt.h>
#include <hipblaslt/hipblaslt-ext.hpp>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <tuple>
#include <vector>

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "%s:%d %s: %s\n", __FILE__, __LINE__, #x, hipGetErrorString(e_)); exit(1); } } while (0)
#define CHECK_BLAS(x) do { hipblasStatus_t s_ = (x); if (s_ != HIPBLAS_STATUS_SUCCESS) { \
  fprintf(stderr, "%s:%d %s: hipblas status %d\n", __FILE__, __LINE__, #x, (int)s_); exit(1); } } while (0)

// N(0, sigma^2) from a counter hash (Box-Muller), rounded to fp16
__global__ void fill_normal(__half* p, int64_t n, float sigma, unsigned seed) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  auto mix = [](uint64_t z) {
    z += 0x9E3779B97F4A7C15ull; z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; return z ^ (z >> 31);
  };
  const uint64_t h = mix((uint64_t)i * 2654435761ull + ((uint64_t)seed << 32));
  const float u1 = ((unsigned)(h >> 40) + 1.0f) * (1.0f / 16777217.0f);
  const float u2 = (unsigned)((h >> 8) & 0xFFFFFF) * (1.0f / 16777216.0f);
  p[i] = __float2half(sigma * sqrtf(-2.0f * logf(u1)) * cosf(6.28318530718f * u2));
}

struct Layer {
  std::string name;
  int64_t T, out, in;
  __half *W = nullptr, *X = nullptr, *Y = nullptr;
};

struct Problem {
  hipblasLtMatmulDesc_t desc;
  hipblasLtMatrixLayout_t a, b, c;
};

static Problem make_problem(int64_t T, int64_t out, int64_t in) {
  // column-major view: Y^T [out x T] = W^T' ... i.e. A = W stored [in x out] column-major, used
  // transposed; B = X stored [in x T] column-major; C = D = Y stored [out x T] column-major
  Problem p;
  CHECK_BLAS(hipblasLtMatmulDescCreate(&p.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F));
  hipblasOperation_t ta = HIPBLAS_OP_T, tb = HIPBLAS_OP_N;
  CHECK_BLAS(hipblasLtMatmulDescSetAttribute(p.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &ta, sizeof(ta)));
  CHECK_BLAS(hipblasLtMatmulDescSetAttribute(p.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &tb, sizeof(tb)));
  CHECK_BLAS(hipblasLtMatrixLayoutCreate(&p.a, HIP_R_16F, in, out, in));
  CHECK_BLAS(hipblasLtMatrixLayoutCreate(&p.b, HIP_R_16F, in, T, in));
  CHECK_BLAS(hipblasLtMatrixLayoutCreate(&p.c, HIP_R_16F, out, T, out));
  return p;
}

int main(int argc, char** argv) {
  int iters = 50, warmup = 10, candidates = 128;
  bool all = false;
  std::vector<Layer> layers;
  for (int i = 1; i < argc; ++i) {
    if (!strcmp(argv[i], "--iters") && i + 1 < argc) iters = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--warmup") && i + 1 < argc) warmup = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--candidates") && i + 1 < argc) candidates = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--all")) all = true;
    else {
      Layer L;
      char name[64];
      long long T, out, in;
      if (sscanf(argv[i], "%63[^:]:%lld:%lld:%lld", name, &T, &out, &in) != 4 || T <= 0 || out <= 0 || in <= 0) {
        fprintf(stderr, "bad layer spec '%s' (want name:T:out:in)\n", argv[i]);
        return 2;
      }
      L.name = name; L.T = T; L.out = out; L.in = in;
      layers.push_back(L);
    }
  }
  if (layers.empty() || iters < 1 || warmup < 0 || candidates < 1) {
    fprintf(stderr, "usage: bench_dense_gemm [--iters N] [--warmup W] [--candidates C] [--all] name:T:out:in ...\n");
    return 2;
  }
  CHECK_HIP(hipSetDevice(0));
  hipStream_t st;
  CHECK_HIP(hipStreamCreate(&st));
  hipblasLtHandle_t h;
  CHECK_BLAS(hipblasLtCreate(&h));
  const size_t ws_bytes = 128ull << 20;
  void* ws = nullptr;
  CHECK_HIP(hipMalloc(&ws, ws_bytes));
  unsigned seed = 1;
  for (auto& L : layers) {
    CHECK_HIP(hipMalloc(&L.W, (size_t)L.out * L.in * 2));
    CHECK_HIP(hipMalloc(&L.X, (size_t)L.T * L.in * 2));
    CHECK_HIP(hipMalloc(&L.Y, (size_t)L.T * L.out * 2));
    const int64_t nw = L.out * L.in, nx = L.T * L.in;
    fill_normal<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>(L.W, nw, 0.02f, seed++);
    fill_normal<<<(unsigned)((nx + 255) / 256), 256, 0, st>>>(L.X, nx, 1.0f, seed++);
  }
  CHECK_HIP(hipStreamSynchronize(st));

  const float alpha = 1.0f, beta = 0.0f;
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  auto run = [&](const Problem& p, const Layer& L, const hipblasLtMatmulAlgo_t& algo) {
    return hipblasLtMatmul(h, p.desc, &alpha, L.W, p.a, L.X, p.b, &beta, L.Y, p.c, L.Y, p.c, &algo, ws, ws_bytes, st);
  };
  auto time_algo = [&](const Problem& p, const Layer& L, const hipblasLtMatmulAlgo_t& algo, int warm, int n) -> double {
    for (int i = 0; i < warm; ++i)
      if (run(p, L, algo) != HIPBLAS_STATUS_SUCCESS) return -1.0;
    CHECK_HIP(hipEventRecord(e0, st));
    for (int i = 0; i < n; ++i)
      if (run(p, L, algo) != HIPBLAS_STATUS_SUCCESS) return -1.0;
    CHECK_HIP(hipEventRecord(e1, st));
    CHECK_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
    return (double)ms / n;
  };

  // ---- search, once per distinct shape
  struct Choice { hipblasLtMatmulAlgo_t algo; double ms; int tried, index; std::string kernel; double heuristic_first_ms; };
  std::map<std::tuple<int64_t, int64_t, int64_t>, Choice> chosen;
  std::map<std::tuple<int64_t, int64_t, int64_t>, Problem> problems;
  for (const auto& L : layers) {
    const auto key = std::make_tuple(L.T, L.out, L.in);
    if (chosen.count(key)) continue;
    Problem p = make_problem(L.T, L.out, L.in);
    problems[key] = p;
    std::vector<hipblasLtMatmulHeuristicResult_t> cand((size_t)candidates);
    hipblasLtMatmulPreference_t pref;
    CHECK_BLAS(hipblasLtMatmulPreferenceCreate(&pref));
    CHECK_BLAS(hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &ws_bytes, sizeof(ws_bytes)));
    int got = 0;
    CHECK_BLAS(hipblasLtMatmulAlgoGetHeuristic(h, p.desc, p.a, p.b, p.c, p.c, pref, candidates, cand.data(), &got));
    cand.resize((size_t)got);
    if (all) {
      std::vector<hipblasLtMatmulHeuristicResult_t> every;
      if (hipblaslt_ext::getAllAlgos(h, hipblaslt_ext::GemmType::HIPBLASLT_GEMM, HIPBLAS_OP_T, HIPBLAS_OP_N, HIP_R_16F,
                                     HIP_R_16F, HIP_R_16F, HIP_R_16F, HIPBLAS_COMPUTE_32F, every) == HIPBLAS_STATUS_SUCCESS) {
        for (auto& r : every) {
          size_t need = 0;
          if (hipblaslt_ext::matmulIsAlgoSupported(h, p.desc, &alpha, p.a, p.b, &beta, p.c, p.c, r.algo, need) ==
                  HIPBLAS_STATUS_SUCCESS && need <= ws_bytes)
            cand.push_back(r);
        }
      }
    }
    if (cand.empty()) { fprintf(stderr, "no hipBLASLt algorithm for %lld x %lld x %lld\n", (long long)L.T, (long long)L.out, (long long)L.in); return 1; }
    // first pass: short timing of every candidate; second pass: the best few again, longer
    std::vector<std::pair<double, size_t>> t;
    double first = -1.0;
    for (size_t i = 0; i < cand.size(); ++i) {
      const double ms = time_algo(p, L, cand[i].algo, 2, 5);
      if (i == 0) first = ms;
      if (ms > 0) t.push_back({ms, i});
    }
    std::sort(t.begin(), t.end());
    Choice best{};
    best.ms = 1e30; best.tried = (int)t.size(); best.heuristic_first_ms = first;
    for (size_t k = 0; k < t.size() && k < 6; ++k) {
      const double ms = time_algo(p, L, cand[t[k].second].algo, 5, 30);
      if (ms > 0 && ms < best.ms) { best.ms = ms; best.algo = cand[t[k].second].algo; }
    }
    best.index = hipblaslt_ext::getIndexFromAlgo(best.algo);
    best.kernel = hipblaslt_ext::getKernelNameFromAlgo(h, best.algo);
    chosen[key] = best;
    CHECK_BLAS(hipblasLtMatmulPreferenceDestroy(pref));
  }

  // ---- measurement: the layers in turn, pass after pass, events around every GEMM
  const int passes = warmup + iters;
  std::vector<std::vector<hipEvent_t>> ev(layers.size());
  for (auto& v : ev) {
    v.resize((size_t)2 * iters);
    for (auto& e : v) CHECK_HIP(hipEventCreate(&e));
  }
  for (int it = 0; it < passes; ++it)
    for (size_t l = 0; l < layers.size(); ++l) {
      const auto key = std::make_tuple(layers[l].T, layers[l].out, layers[l].in);
      const bool rec = it >= warmup;
      if (rec) CHECK_HIP(hipEventRecord(ev[l][(size_t)2 * (it - warmup)], st));
      CHECK_BLAS(run(problems[key], layers[l], chosen[key].algo));
      if (rec) CHECK_HIP(hipEventRecord(ev[l][(size_t)2 * (it - warmup) + 1], st));
    }
  CHECK_HIP(hipStreamSynchronize(st));

  int ver = 0;
  hipblasLtGetVersion(h, &ver);
  printf("{\"library\": \"hipBLASLt %d\", \"search\": \"%s\", \"iters\": %d, \"warmup\": %d, \"layers\": [",
         ver, all ? "heuristic candidates + all supported algorithms, timed" : "heuristic candidates, timed", iters, warmup);
  for (size_t l = 0; l < layers.size(); ++l) {
    const Layer& L = layers[l];
    const auto key = std::make_tuple(L.T, L.out, L.in);
    std::vector<double> ms((size_t)iters);
    double sum = 0;
    for (int i = 0; i < iters; ++i) {
      float m = 0.f;
      CHECK_HIP(hipEventElapsedTime(&m, ev[l][(size_t)2 * i], ev[l][(size_t)2 * i + 1]));
      ms[(size_t)i] = m; sum += m;
    }
    std::sort(ms.begin(), ms.end());
    const Choice& c = chosen[key];
    printf("%s{\"layer\": \"%s\", \"tokens\": %lld, \"out\": %lld, \"in\": %lld, \"median_ms\": %.6f, \"mean_ms\": %.6f, "
           "\"min_ms\": %.6f, \"candidates_timed\": %d, \"algo_index\": %d, \"kernel\": \"%s\", "
           "\"search_best_ms\": %.6f, \"heuristic_first_ms\": %.6f}",
           l ? ", " : "", L.name.c_str(), (long long)L.T, (long long)L.out, (long long)L.in, ms[(size_t)iters / 2],
           sum / iters, ms[0], c.tried, c.index, c.kernel.c_str(), c.ms, c.heuristic_first_ms);
  }
  printf("]}\n");
  fflush(stdout);
  return 0;
}
