"""MI355X-native hot path of DSGD-CECA (arXiv 2306.00256): thin Python binding over libceca.so.

Every step of the path runs in the HIP kernels behind the C ABI of include/ceca.h; this package only
marshals arguments.  PyTorch supplies device memory and streams.  There is no CPU fallback: loading
fails if the library has not been built (python -m paper_2306_00256_amd.build).
"""
from .binding import (  # noqa: F401
    CecaError,
    Loss,
    Mix,
    Round,
    ceca_average,
    ceca_describe_step_launch,
    ceca_gossip_round,
    ceca_gossip_rounds,
    ceca_graph_rounds,
    ceca_mix_rounds,
    ceca_reset_options,
    ceca_schedule,
    ceca_set_option,
    ceca_stream_probe,
    ceca_tau,
    ceca_topology_round,
    ceca_state_consensus,
    consensus_error,
    consensus_error_noalloc,
    consensus_error_workspace_bytes,
    dsgd_ceca_run,
    dsgd_ceca_run_workspace_bytes,
    dsgd_ceca_step,
    dsgd_ceca_steps,
    dsgd_ceca_workspace_bytes,
    lib,
    library_path,
)
