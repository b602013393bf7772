#include "schedule.h"

namespace ceca {

int32_t tau_of(int32_t n) {
  int32_t t = 0;
  for (uint32_t m = (uint32_t)(n - 1); m; m >>= 1) ++t;
  return t;
}

void fill_round(int32_t n, int32_t r, int32_t port, ceca_round_t* out) {
  const int32_t tau = tau_of(n);
  const uint32_t nm1 = (uint32_t)(n - 1);
  // walk the digits of n-1 from the top: n_{q+1} = 2 n_q + delta_q (Eq. (3))
  int32_t nr = 0;
  for (int32_t q = 0; q < r; ++q) nr = 2 * nr + (int32_t)((nm1 >> (tau - 1 - q)) & 1u);
  const int32_t delta = (int32_t)((nm1 >> (tau - 1 - r)) & 1u);
  out->n = n;
  out->tau = tau;
  out->r = r;
  out->port = port;
  out->delta = delta;
  out->n_r = nr;
  out->shift = (port == 2) ? nr + delta : 2 * nr + 1;
  out->exchange_y = delta ? 0 : 1;
  const int32_t den = 2 * nr + 1;
  if (delta) {            // x travels: a = 1/2, b = n_r / (2 n_r + 1)
    out->a_num = 1;  out->a_den = 2;
    out->b_num = nr; out->b_den = den;
  } else {                // y travels: a = (n_r + 1) / (2 n_r + 1), b = 1/2
    out->a_num = nr + 1; out->a_den = den;
    out->b_num = 1;      out->b_den = 2;
  }
  out->a = (float)((double)out->a_num / (double)out->a_den);
  out->a_peer = (float)((double)(out->a_den - out->a_num) / (double)out->a_den);
  out->b = (float)((double)out->b_num / (double)out->b_den);
  out->b_peer = (float)((double)(out->b_den - out->b_num) / (double)out->b_den);
}

bool fill_topology(int32_t kind, int32_t n, int32_t k, ceca_mix_t* out) {
  *out = ceca_mix_t{};
  if (n < 1 || k < 0) return false;
  const int32_t tau = tau_of(n);
  double w = 0.0;
  switch (kind) {
    case CECA_TOPO_RING:
      if (n == 2) { out->m = 1; out->shift[0] = 1; w = 0.5; }
      else if (n > 2) { out->m = 2; out->shift[0] = 1; out->shift[1] = n - 1; w = 1.0 / 3.0; }
      break;
    case CECA_TOPO_STATIC_EXP:
      if (tau > CECA_MIX_MAX) return false;
      out->m = tau;
      w = 1.0 / (double)(tau + 1);
      for (int32_t j = 0; j < tau; ++j) out->shift[j] = (int32_t)(1u << j);
      break;
    case CECA_TOPO_ONE_PEER_EXP:
      if (tau > 0) { out->m = 1; out->shift[0] = (int32_t)(1u << (k % tau)); w = 0.5; }
      break;
    default:
      return false;
  }
  double rest = 1.0;
  for (int32_t j = 0; j < out->m; ++j) {
    out->w[j] = (float)w;
    rest -= (double)out->w[j];
  }
  out->w_self = (float)rest;
  return true;
}

}  // namespace ceca
