"""CPU oracle for the DSGD-CECA hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 restatement of what the paper defines (CECA Sec. 3,
DSGD-CECA Sec. 4.1).  It shares no code with the HIP library and must never be
imported by it; only tests, the smoke check and the benchmark's CPU-baseline leg
may use it.

Pin status (see tests/test_oracle_*.py):
  schedule (tau, delta_r, n_r, peers, weights) ... pinned by the paper's n=6 example,
      n_tau = n-1, permutation / involution structure
  gossip round (per-agent and dense W form) ...... pinned by the paper's printed n=6 value
      tables and coefficient matrices, the window invariants (Eq. 4 and its 1-port
      analogue), and the exact tau-round product of the matrix-consensus lemma for
      every n <= 64
  mixing matrices W, W_g ........................ pinned by Lemma 4.1 (row sums, norm,
      commutation) and by agreement with the per-agent form
  DSGD-CECA step ................................. pinned by the mean recursion of the
      averaged-variables lemma, the two codings agreeing, and the noise-free
      quadratic closed form; a full trajectory is not printed by the paper, so
      *trajectory parity is unpinned by the paper* beyond those properties
  losses ......................................... not the paper's (they come with the
      benchmark configurations): pinned by finite differences and closed forms
  noise generator ................................ defined by this build, not by the paper:
      pinned only statistically (mean, variance, independence) -- *parity unpinned*
      as to the specific stream
  consensus metrics .............................. pinned by closed forms on hand-made inputs
  comparison topologies (ring, static / one-peer exponential gossip) ... defined by the works
      the paper cites, not by the paper: pinned by stochasticity, three codings agreeing
      (per agent, dense, circular convolution), one-hot direction checks, the power-of-two
      exact-averaging property and its equality with CECA; *parity unpinned by the paper*
  gossip over arbitrary graphs (Metropolis weights; hypercube, torus, grid of Table 1) ... textbook
      definitions, not the paper's: pinned by hand-made weight matrices, closed-form spectra, exact
      averaging of the one-peer hypercube, equality with the circulant oracle on a ring;
      *parity unpinned by the paper*
"""
