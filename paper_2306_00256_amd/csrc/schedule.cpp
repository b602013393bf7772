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

}  // namespace ceca
