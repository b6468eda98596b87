// Transport optimisation of the paper's Section 2.2 (Eq. 5), host only: which p layers
// become all-streaming.  See include/zz.h for the contract.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "zz.h"

extern "C" int zz_transport_select(const float *alpha, int n_layers, int n_heads, float sparsity, float omega,
                                   uint8_t *layer_is_streaming, double *loss) {
  if (!alpha || !layer_is_streaming || n_layers < 1 || n_heads < 1) return ZZ_EINVAL;
  if (!(sparsity >= 0.f && sparsity <= 1.f) || !(omega >= 0.f && omega <= 1.f)) return ZZ_ERANGE;
  // p / L = s must hold exactly (Section 2.2): s * L has to be a whole number of layers
  const double pl = (double)sparsity * (double)n_layers;
  if (std::fabs(pl - std::nearbyint(pl)) > 1e-4) return ZZ_ERANGE;
  const size_t n = (size_t)n_layers * n_heads;
  for (size_t t = 0; t < n; ++t)
    if (!(alpha[t] >= 0.f && alpha[t] <= 1.f)) return ZZ_ERANGE;

  // Step 1: the starting point.  The heads of smallest alpha, round(sparsity*L*H) of them,
  // are streaming heads (ties by index).
  const size_t n_stream = (size_t)std::llround(std::nearbyint(pl) * (double)n_heads);
  std::vector<size_t> order(n);
  std::iota(order.begin(), order.end(), (size_t)0);
  std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return alpha[a] < alpha[b]; });
  std::vector<uint8_t> head_streams(n, 0);
  for (size_t r = 0; r < n_stream; ++r) head_streams[order[r]] = 1;

  // Step 2: per layer, what it costs to make it all-streaming (its retrieval heads turn) and
  // what making it all-retrieval gains (its streaming heads turn, weight omega).
  std::vector<double> to_streaming(n_layers, 0.0), to_retrieval(n_layers, 0.0), key(n_layers);
  for (int i = 0; i < n_layers; ++i) {
    for (int j = 0; j < n_heads; ++j) {
      const size_t t = (size_t)i * n_heads + j;
      (head_streams[t] ? to_retrieval[i] : to_streaming[i]) += (double)alpha[t];
    }
    key[i] = to_streaming[i] + (double)omega * to_retrieval[i];
  }

  // Step 3: the p layers of smallest key.
  const int p = (int)std::llround(pl);
  std::vector<int> layers(n_layers);
  std::iota(layers.begin(), layers.end(), 0);
  std::stable_sort(layers.begin(), layers.end(), [&](int a, int b) { return key[a] < key[b]; });
  std::fill(layer_is_streaming, layer_is_streaming + n_layers, (uint8_t)0);
  for (int r = 0; r < p; ++r) layer_is_streaming[layers[r]] = 1;
  if (loss) {
    double total = 0.0;
    for (int i = 0; i < n_layers; ++i)
      total += layer_is_streaming[i] ? to_streaming[i] : -(double)omega * to_retrieval[i];
    *loss = total;
  }
  return ZZ_OK;
}
