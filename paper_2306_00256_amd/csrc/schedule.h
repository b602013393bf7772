// Host-side CECA round schedule (integer exact).  Sec. 3.1 Eqs. (2), (3), (5), (6); Sec. 3.2 Eq. (7);
// weights of Algorithm 1 (Sec. 4.1).
#pragma once
#include <cstdint>

#include "ceca.h"

namespace ceca {

// Bit length of n-1: the number of rounds tau = ceil(log2 n) without floating point.
int32_t tau_of(int32_t n);

// Fills `out` for round r of an n-agent schedule.  Expects n >= 2, 0 <= r < tau, port in {1, 2},
// and even n for port 1 (the caller validates).
void fill_round(int32_t n, int32_t r, int32_t port, ceca_round_t* out);

// Row that row i receives from in the round described by `rd`.
inline int32_t peer_of(const ceca_round_t& rd, int32_t i) {
  int64_t j;
  if (rd.port == 2) {
    j = (int64_t)i - rd.shift;
  } else {
    // 0-based even rows are the paper's odd agents: they look ahead, the others look back
    j = (i & 1) ? (int64_t)i - rd.shift : (int64_t)i + rd.shift;
  }
  j %= rd.n;
  if (j < 0) j += rd.n;
  return (int32_t)j;
}

// Round k of a comparison topology (ring, static / one-peer exponential gossip).  Expects n >= 1,
// k >= 0 and a known kind; returns false otherwise.
bool fill_topology(int32_t kind, int32_t n, int32_t k, ceca_mix_t* out);

}  // namespace ceca
