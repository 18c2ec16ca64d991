// Head partition model (Section III-D: Algorithm 2 and the latency estimates of the two head
// kinds).  Host arithmetic only; part of the library so that callers of the C ABI can pick the
// head split from their own measurements.
#include <cmath>

#include "../../include/gformer.h"

namespace {

bool positive(double x) { return std::isfinite(x) && x > 0.0; }
bool non_negative(double x) { return std::isfinite(x) && x >= 0.0; }

}  // namespace

extern "C" {

gf_status gformer_partition_balance(const gformer_partition_inputs* in, double* p_prime,
                                    double* latency) {
  if (!in || !p_prime) return GF_ERR_INVALID_ARG;
  if (in->struct_size != sizeof(gformer_partition_inputs) || in->reserved0 != 0)
    return GF_ERR_INVALID_ARG;
  if (!positive(in->size) || !positive(in->perf0) || !positive(in->perf1)) return GF_ERR_INVALID_ARG;
  if (!non_negative(in->flops_per0) || !non_negative(in->flops_per1)) return GF_ERR_INVALID_ARG;
  if (in->flops_per0 == 0.0 && in->flops_per1 == 0.0) return GF_ERR_INVALID_ARG;
  if (!(in->p >= 0.0 && in->p <= 1.0)) return GF_ERR_INVALID_ARG;
  // seconds per unit on each side; equal latencies <=> p' c0 = (1 - p') c1
  const double c0 = in->flops_per0 / in->perf0;
  const double c1 = in->flops_per1 / in->perf1;
  const double pp = c1 / (c0 + c1);
  *p_prime = pp;
  if (latency) {
    latency[0] = in->p * in->size * c0;
    latency[1] = (1.0 - in->p) * in->size * c1;
    latency[2] = pp * in->size * c0;
    latency[3] = (1.0 - pp) * in->size * c1;
  }
  return GF_OK;
}

gf_status gformer_partition_heads(int B, int H, int N, int E, int W, double perf_sparse,
                                  double perf_linear, int flop_model, int* H0, double* latency) {
  if (!H0) return GF_ERR_INVALID_ARG;
  if (B < 1 || H < 1 || N < 1 || E < 1 || W < 1) return GF_ERR_INVALID_ARG;
  if (flop_model != GF_FLOPS_PAPER && flop_model != GF_FLOPS_PER_HEAD) return GF_ERR_INVALID_ARG;
  if (!positive(perf_sparse) || !positive(perf_linear)) return GF_ERR_INVALID_ARG;
  const double b = B, n = N, e = E, w = W;
  int best = 0;
  double best_gap = INFINITY, best_s = 0.0, best_l = 0.0;
  for (int h0 = 0; h0 <= H; ++h0) {
    const double hs = h0, hl = H - h0;
    const double flops_s = 2.0 * b * hs * e * n * w + 3.0 * b * hs * n * w;
    const double width = hl * e;
    const double flops_l = flop_model == GF_FLOPS_PAPER ? 8.0 * b * n * width * width
                                                        : 8.0 * b * n * hl * e * e;
    const double ls = flops_s / perf_sparse, ll = flops_l / perf_linear;
    const double gap = std::fabs(ls - ll);
    if (gap < best_gap) {
      best_gap = gap;
      best = h0;
      best_s = ls;
      best_l = ll;
    }
  }
  *H0 = best;
  if (latency) {
    latency[0] = best_s;
    latency[1] = best_l;
  }
  return GF_OK;
}

}  // extern "C"
