// A client of the C ABI that uses nothing but the HIP runtime and artopk.h: no
// Python, no PyTorch.  It runs two AR-Topk steps (Alg. 1 loop body with the error
// feedback of Sec. II-C) for W workers under the round-robin leader rule and
// checks every output against a plain host computation written here.
//
//   build:  hipcc -O2 --offload-arch=gfx950 -I include tests/abi_client/abi_client.cpp \
//                 -L paper_2312_02493_amd -lartopk -Wl,-rpath,$PWD/paper_2312_02493_amd \
//                 -o tests/abi_client/abi_client        (python -m paper_2312_02493_amd.build does this)
//   run:    tests/abi_client/abi_client [N] [W] [k] [segments]   (exit code 0 = all outputs identical;
//           with segments > 1 the selection is per segment, k split in proportion to the sizes)

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "artopk.h"

#define HIP_OK(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) {                                                               \
      std::fprintf(stderr, "%s failed: %s\n", #expr, hipGetErrorString(e_));              \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)

#define ART_OK(ctx, expr)                                                                 \
  do {                                                                                    \
    int rc_ = (expr);                                                                     \
    if (rc_ != ARTOPK_OK) {                                                               \
      std::fprintf(stderr, "%s returned %d: %s\n", #expr, rc_, artopk_last_error(ctx));   \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)

static uint32_t bits_of(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  return u;
}

// A small generator of its own (xorshift), mapped to roughly Laplace-shaped values with ties.
static float draw(uint64_t& s) {
  s ^= s << 13;
  s ^= s >> 7;
  s ^= s << 17;
  const double u = (double)((s >> 11) & 0xfffff) / 1048576.0;       // [0, 1)
  const double mag = -1e-2 * std::log(1.0 - 0.999999 * u);
  const float v = (float)(((s >> 40) & 1) ? -mag : mag);
  return ((s >> 45) % 10 == 0) ? (float)((int)(v * 1024.0f)) / 1024.0f : v;  // a tenth on a coarse grid
}

int main(int argc, char** argv) {
  const int64_t n = argc > 1 ? std::atoll(argv[1]) : 200003;
  const int32_t w = argc > 2 ? std::atoi(argv[2]) : 3;
  int64_t k = argc > 3 ? std::atoll(argv[3]) : (n + 99) / 100;
  const int32_t nseg = argc > 4 ? std::atoi(argv[4]) : 1;
  const bool short_routes = argc > 5 && std::atoi(argv[5]) != 0;  // take the long-vector routes on this short one
  if (n < 1 || w < 1 || w > ARTOPK_MAX_WORKERS || k < 1 || k > n || nseg < 1 || nseg > n) {
    std::fprintf(stderr, "usage: abi_client [N] [W] [k] [segments] [long-vector routes: 0|1]\n");
    return 2;
  }
  // segment table (host memory): equal parts, every part keeping its share of k (at least one)
  std::vector<int64_t> seg_off(nseg + 1), seg_k(nseg);
  for (int s = 0; s <= nseg; ++s) seg_off[s] = n * s / nseg;
  if (nseg > 1) {
    const int64_t k_asked = k;
    k = 0;
    for (int s = 0; s < nseg; ++s) {
      const int64_t size = seg_off[s + 1] - seg_off[s];
      seg_k[s] = std::max<int64_t>(1, std::min<int64_t>(size, k_asked * size / n));
      k += seg_k[s];
    }
  } else {
    seg_k[0] = k;
  }

  std::vector<std::vector<float>> g(w, std::vector<float>(n)), res(w, std::vector<float>(n, 0.0f));
  std::vector<float*> g_dev(w), res_dev(w);
  for (int r = 0; r < w; ++r) {
    HIP_OK(hipMalloc(&g_dev[r], n * sizeof(float)));
    HIP_OK(hipMalloc(&res_dev[r], n * sizeof(float)));
    HIP_OK(hipMemset(res_dev[r], 0, n * sizeof(float)));
  }
  int32_t* idx_dev;
  float *vals_dev, *sum_dev, *update_dev;
  int32_t* leader_dev;
  HIP_OK(hipMalloc(&idx_dev, k * sizeof(int32_t)));
  HIP_OK(hipMalloc(&vals_dev, (size_t)w * k * sizeof(float)));
  HIP_OK(hipMalloc(&sum_dev, k * sizeof(float)));
  HIP_OK(hipMalloc(&update_dev, n * sizeof(float)));
  HIP_OK(hipMalloc(&leader_dev, sizeof(int32_t)));

  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  artopk_ctx* ctx = nullptr;
  if (artopk_create(&ctx, w, n, k, nseg, stream) != ARTOPK_OK) {
    std::fprintf(stderr, "artopk_create failed\n");
    return 2;
  }
  if (short_routes) {
    ART_OK(ctx, artopk_set_option(ctx, ARTOPK_OPT_GUESS_MIN_N, 4096));
    ART_OK(ctx, artopk_set_option(ctx, ARTOPK_OPT_UPDATE_TILES_MIN_N, 1));
  }

  uint64_t seed = 0x9e3779b97f4a7c15ull;
  long mismatches = 0;
  for (uint64_t step = 1; step <= 2; ++step) {
    for (int r = 0; r < w; ++r) {
      for (int64_t i = 0; i < n; ++i) g[r][i] = draw(seed);
      HIP_OK(hipMemcpyAsync(g_dev[r], g[r].data(), n * sizeof(float), hipMemcpyHostToDevice, stream));
    }
    ART_OK(ctx, artopk_step(ctx, g_dev.data(), res_dev.data(), w, n, nseg, nseg > 1 ? seg_off.data() : nullptr,
                            nseg > 1 ? seg_k.data() : nullptr, k, ARTOPK_STAR, step, 0, leader_dev, nullptr, idx_dev,
                            vals_dev, sum_dev, update_dev));
    ART_OK(ctx, artopk_status(ctx));  // synchronises the stream

    // ---- the same step on the host, straight from the definitions -------------------------
    const int leader = (int)(step % (uint64_t)w);
    std::vector<std::vector<float>> acc(w, std::vector<float>(n));
    for (int r = 0; r < w; ++r)
      for (int64_t i = 0; i < n; ++i) acc[r][i] = g[r][i] + res[r][i];
    std::vector<int32_t> order(n);
    for (int64_t i = 0; i < n; ++i) order[i] = (int32_t)i;
    const std::vector<float>& lead = acc[leader];
    std::vector<int32_t> idx;
    for (int s = 0; s < nseg; ++s) {  // per segment: larger magnitude first, then lower index; keep seg_k[s]
      std::sort(order.begin() + seg_off[s], order.begin() + seg_off[s + 1], [&](int32_t a, int32_t b) {
        const uint32_t ka = bits_of(lead[a]) & 0x7fffffffu, kb = bits_of(lead[b]) & 0x7fffffffu;
        return ka != kb ? ka > kb : a < b;
      });
      idx.insert(idx.end(), order.begin() + seg_off[s], order.begin() + seg_off[s] + seg_k[s]);
    }
    std::sort(idx.begin(), idx.end());
    std::vector<float> sum(k), update(n, 0.0f);
    for (int64_t m = 0; m < k; ++m) {
      float s = acc[0][idx[m]];
      for (int r = 1; r < w; ++r) s = s + acc[r][idx[m]];
      sum[m] = s;
      update[idx[m]] = s;
    }
    for (int r = 0; r < w; ++r) {
      res[r] = acc[r];
      for (int64_t m = 0; m < k; ++m) res[r][idx[m]] = 0.0f;
    }

    // ---- compare, bit for bit ---------------------------------------------------------------
    int32_t leader_got = -1;
    std::vector<int32_t> idx_got(k);
    std::vector<float> sum_got(k), update_got(n), vals_got((size_t)w * k), res_got(n);
    HIP_OK(hipMemcpy(&leader_got, leader_dev, sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(idx_got.data(), idx_dev, k * sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(sum_got.data(), sum_dev, k * sizeof(float), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(update_got.data(), update_dev, n * sizeof(float), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(vals_got.data(), vals_dev, (size_t)w * k * sizeof(float), hipMemcpyDeviceToHost));
    long bad = (leader_got != leader);
    for (int64_t m = 0; m < k; ++m) bad += idx_got[m] != idx[m];
    for (int64_t m = 0; m < k; ++m) bad += bits_of(sum_got[m]) != bits_of(sum[m]);
    for (int64_t i = 0; i < n; ++i) bad += bits_of(update_got[i]) != bits_of(update[i]);
    for (int r = 0; r < w; ++r) {
      for (int64_t m = 0; m < k; ++m) bad += bits_of(vals_got[(size_t)r * k + m]) != bits_of(acc[r][idx[m]]);
      HIP_OK(hipMemcpy(res_got.data(), res_dev[r], n * sizeof(float), hipMemcpyDeviceToHost));
      for (int64_t i = 0; i < n; ++i) bad += bits_of(res_got[i]) != bits_of(res[r][i]);
    }
    std::printf("step %llu: leader %d, k %lld of %lld, %ld mismatching outputs\n", (unsigned long long)step, leader_got,
                (long long)k, (long long)n, bad);
    mismatches += bad;
  }

  ART_OK(ctx, artopk_destroy(ctx));
  for (int r = 0; r < w; ++r) {
    HIP_OK(hipFree(g_dev[r]));
    HIP_OK(hipFree(res_dev[r]));
  }
  HIP_OK(hipFree(idx_dev));
  HIP_OK(hipFree(vals_dev));
  HIP_OK(hipFree(sum_dev));
  HIP_OK(hipFree(update_dev));
  HIP_OK(hipFree(leader_dev));
  HIP_OK(hipStreamDestroy(stream));
  std::printf(mismatches == 0 ? "abi_client: ok\n" : "abi_client: FAILED\n");
  return mismatches == 0 ? 0 : 1;
}
