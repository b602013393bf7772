"""ctypes binding of include/ceca.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libceca.so")

CECA_OK, CECA_EINVAL, CECA_EODD1P, CECA_EWORKSPACE, CECA_EHIP = 0, -1, -2, -3, -4
LOSS_LSQ, LOSS_LOGISTIC, LOSS_QUAD_CENTER, LOSS_GRADIENT = 0, 1, 2, 3
# options of the test and measurement interface (include/ceca_test.h)
OPT_SEGMENT, OPT_ROWS, OPT_BAND, OPT_WG_PER_CU, OPT_ONEPASS, OPT_AGENTS_PER_WG, OPT_CONS_SINGLE_PASS, OPT_XCD_TILE_ORDER, OPT_TILE_THREADS = 1, 2, 3, 4, 5, 7, 8, 9, 10
OPT_GRAPH_STAGE, OPT_CHUNKED_GRADIENT, OPT_CONS_STRIPS, OPT_PROBE_WAVES, OPT_LEAN_TILES, OPT_PROBE_VARIANT, OPT_HALF_STEP_RUN = 11, 12, 13, 14, 15, 16, 17
TOPO_RING, TOPO_STATIC_EXP, TOPO_ONE_PEER_EXP = 0, 1, 2
MIX_MAX = 16

EXPORTS = (
    "ceca_tau", "ceca_schedule", "ceca_gossip_round", "ceca_gossip_rounds", "ceca_average", "dsgd_ceca_workspace_bytes", "dsgd_ceca_step", "dsgd_ceca_steps", "dsgd_ceca_run_workspace_bytes", "dsgd_ceca_run",
    "consensus_error_workspace_bytes", "consensus_error", "consensus_error_noalloc", "ceca_state_consensus", "ceca_topology_round", "ceca_mix_rounds", "ceca_graph_rounds", "ceca_last_error", "ceca_last_hip_error",
)
# include/ceca_test.h: launch-shape overrides and probe kernels for tests and measurement, not the product ABI
TEST_EXPORTS = ("ceca_set_option", "ceca_reset_options", "ceca_stream_probe", "ceca_describe_step_launch")


class CecaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ceca error {code}: {msg}")
        self.code = code


class Round(C.Structure):
    """ceca_round_t"""
    _fields_ = [(k, C.c_int32) for k in ("n", "tau", "r", "port", "delta", "n_r", "shift", "exchange_y",
                                         "a_num", "a_den", "b_num", "b_den")] + \
               [(k, C.c_float) for k in ("a", "a_peer", "b", "b_peer")]


class Loss(C.Structure):
    """ceca_loss_t"""
    _fields_ = [("kind", C.c_int32), ("N", C.c_int32), ("B", C.c_int32), ("seed", C.c_uint32), ("k", C.c_uint32),
                ("noise_std", C.c_float), ("grad_scale", C.c_float), ("A", C.c_void_p), ("lda", C.c_int64), ("t", C.c_void_p),
                ("c", C.c_void_p), ("ldc", C.c_int64)]


class Mix(C.Structure):
    """ceca_mix_t"""
    _fields_ = [("m", C.c_int32), ("w_self", C.c_float), ("shift", C.c_int32 * MIX_MAX), ("w", C.c_float * MIX_MAX)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library; raises if it was never built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2306_00256_amd.build`")
        L = C.CDLL(_LIB_PATH)
        L.ceca_tau.argtypes = [C.c_int32]
        L.ceca_tau.restype = C.c_int32
        L.ceca_schedule.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(Round), C.POINTER(C.c_int32)]
        L.ceca_schedule.restype = C.c_int32
        L.ceca_gossip_round.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_int32,
                                        C.c_int32, C.c_void_p]
        L.ceca_gossip_round.restype = C.c_int32
        L.ceca_gossip_rounds.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_int32,
                                         C.c_int32, C.c_void_p]
        L.ceca_gossip_rounds.restype = C.c_int32
        L.dsgd_ceca_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.POINTER(Loss)]
        L.dsgd_ceca_workspace_bytes.restype = C.c_int64
        L.dsgd_ceca_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.POINTER(Loss),
                                     C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                     C.c_void_p]
        L.dsgd_ceca_step.restype = C.c_int32
        L.ceca_average.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.c_void_p]
        L.ceca_average.restype = C.c_int32
        L.dsgd_ceca_steps.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.POINTER(Loss), C.c_float,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.dsgd_ceca_steps.restype = C.c_int32
        L.dsgd_ceca_run_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.POINTER(Loss)]
        L.dsgd_ceca_run_workspace_bytes.restype = C.c_int64
        L.dsgd_ceca_run.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.POINTER(Loss), C.c_void_p,
                                    C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
        L.dsgd_ceca_run.restype = C.c_int32
        L.consensus_error_workspace_bytes.argtypes = [C.c_int32, C.c_int64]
        L.consensus_error_workspace_bytes.restype = C.c_int64
        L.consensus_error.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int64, C.c_void_p]
        L.consensus_error.restype = C.c_int32
        L.consensus_error_noalloc.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.consensus_error_noalloc.restype = C.c_int32
        L.ceca_state_consensus.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                           C.c_int64, C.c_void_p]
        L.ceca_state_consensus.restype = C.c_int32
        L.ceca_topology_round.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(Mix)]
        L.ceca_topology_round.restype = C.c_int32
        L.ceca_mix_rounds.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.POINTER(Mix), C.c_int32,
                                      C.c_int32, C.c_int32, C.c_void_p]
        L.ceca_mix_rounds.restype = C.c_int32
        L.ceca_graph_rounds.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.ceca_graph_rounds.restype = C.c_int32
        L.ceca_stream_probe.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
        L.ceca_stream_probe.restype = C.c_int32
        L.ceca_describe_step_launch.argtypes = [C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                                C.POINTER(C.c_int32)]
        L.ceca_describe_step_launch.restype = C.c_int32
        L.ceca_reset_options.argtypes = []
        L.ceca_reset_options.restype = C.c_int32
        L.ceca_last_error.restype = C.c_char_p
        L.ceca_last_hip_error.restype = C.c_int32
        L.ceca_set_option.argtypes = [C.c_int32, C.c_int32]
        L.ceca_set_option.restype = C.c_int32
        _lib = L
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise CecaError(int(rc), lib().ceca_last_error().decode())
    return int(rc)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = int(stream.cuda_stream)
    return h if h else None


def ceca_tau(n: int) -> int:
    return _check(lib().ceca_tau(n))


def ceca_schedule(n: int, r: int, port: int) -> Tuple[Round, List[int]]:
    """(round description, 0-based receive-from map) of round r."""
    rd = Round()
    peer = (C.c_int32 * max(n, 1))()
    _check(lib().ceca_schedule(n, r, port, C.byref(rd), peer))
    return rd, list(peer)


def ceca_gossip_round(S_in, S_out, n: int, d: int, r: int, port: int, ld: Optional[int] = None, stream=None) -> None:
    """S_in, S_out: device float32 tensors holding 2n rows of ld floats (x rows, then y rows)."""
    ld = int(S_in.stride(0)) if ld is None else ld
    _check(lib().ceca_gossip_round(_ptr(S_in), _ptr(S_out), n, d, ld, r, port, _stream(stream)))


def ceca_gossip_rounds(S_in, S_out, n: int, d: int, rounds: int, port: int, ld: Optional[int] = None,
                       stream=None) -> None:
    """`rounds` gradient-free rounds starting at round 0, fused into one pass."""
    ld = int(S_in.stride(0)) if ld is None else ld
    _check(lib().ceca_gossip_rounds(_ptr(S_in), _ptr(S_out), n, d, ld, rounds, port, _stream(stream)))


def ceca_topology_round(kind: int, n: int, k: int = 0) -> Mix:
    m = Mix()
    _check(lib().ceca_topology_round(kind, n, k, C.byref(m)))
    return m


def ceca_mix_rounds(X_in, X_out, n: int, d: int, specs: Sequence[Mix], rounds: int, k0: int = 0,
                    ld: Optional[int] = None, stream=None) -> None:
    """`rounds` shift-invariant mixing rounds on x alone; round t applies specs[(k0 + t) % len(specs)]."""
    ld = int(X_in.stride(0)) if ld is None else ld
    arr = (Mix * len(specs))(*specs)
    _check(lib().ceca_mix_rounds(_ptr(X_in), _ptr(X_out), n, d, ld, arr, len(specs), k0, rounds, _stream(stream)))


def ceca_graph_rounds(X_in, X_out, n: int, d: int, nbr, w, w_self, rounds: int, k0: int = 0,
                      ld: Optional[int] = None, stream=None) -> None:
    """`rounds` gossip rounds over a graph given as device tables: nbr (period, n, m) int32, w (period, n, m)
    float32, w_self (period, n) float32, all contiguous; round t uses tables[(k0 + t) % period]."""
    ld = int(X_in.stride(0)) if ld is None else ld
    period, _, m = nbr.shape
    _check(lib().ceca_graph_rounds(_ptr(X_in), _ptr(X_out), n, d, ld, _ptr(nbr), _ptr(w), _ptr(w_self), m, period, k0,
                                   rounds, _stream(stream)))


def ceca_average(X_in, X_out, n: int, d: int, port: int, ld: Optional[int] = None, stream=None) -> None:
    """Every row of X_out becomes the mean of the rows of X_in (tau CECA rounds in one pass, x only)."""
    ld = int(X_in.stride(0)) if ld is None else ld
    _check(lib().ceca_average(_ptr(X_in), _ptr(X_out), n, d, ld, port, _stream(stream)))


def dsgd_ceca_workspace_bytes(n: int, d: int, loss: Loss) -> int:
    return _check(lib().dsgd_ceca_workspace_bytes(n, d, C.byref(loss)))


def dsgd_ceca_step(S_in, S_out, n: int, d: int, loss: Loss, batch_idx, lr: float, r: int, port: int,
                   workspace=None, ld: Optional[int] = None, stream=None) -> None:
    ld = int(S_in.stride(0)) if ld is None else ld
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().dsgd_ceca_step(_ptr(S_in), _ptr(S_out), n, d, ld, C.byref(loss), _ptr(batch_idx), lr, r, port,
                                _ptr(workspace), wbytes, _stream(stream)))


def dsgd_ceca_steps(S_in, S_out, n: int, d: int, loss: Loss, lr: float, r0: int, steps: int, port: int,
                    ld: Optional[int] = None, stream=None) -> None:
    """`steps` iterations with the quadratic-centre loss fused into one pass (rounds r0, r0 + 1, ...;
    noise counters loss.k, loss.k + 1, ...)."""
    ld = int(S_in.stride(0)) if ld is None else ld
    _check(lib().dsgd_ceca_steps(_ptr(S_in), _ptr(S_out), n, d, ld, C.byref(loss), lr, r0, steps, port, _stream(stream)))


def dsgd_ceca_run_workspace_bytes(n: int, d: int, loss: Loss) -> int:
    return _check(lib().dsgd_ceca_run_workspace_bytes(n, d, C.byref(loss)))


def dsgd_ceca_run(S_in, S_out, n: int, d: int, loss: Loss, batch_idx, lr: float, r0: int, iters: int, port: int,
                  workspace=None, ld: Optional[int] = None, stream=None) -> None:
    """`iters` iterations with a minibatch loss in one call (batch_idx: iters x n x B int32 on the device)."""
    ld = int(S_in.stride(0)) if ld is None else ld
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().dsgd_ceca_run(_ptr(S_in), _ptr(S_out), n, d, ld, C.byref(loss), _ptr(batch_idx), lr, r0, iters, port,
                               _ptr(workspace), wbytes, _stream(stream)))


def consensus_error_workspace_bytes(n: int, d: int) -> int:
    return _check(lib().consensus_error_workspace_bytes(n, d))


def consensus_error(X, n: int, d: int, out, xbar=None, workspace=None, ld: Optional[int] = None, stream=None) -> None:
    """out: device float64 tensor of 5; see include/ceca.h for its layout."""
    ld = int(X.stride(0)) if ld is None else ld
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().consensus_error(_ptr(X), n, d, ld, _ptr(out), _ptr(xbar), _ptr(workspace), wbytes, _stream(stream)))


def consensus_error_noalloc(X, n: int, d: int, out, xbar=None, ld: Optional[int] = None, stream=None) -> None:
    """consensus_error without a workspace: the partial sums live in the library's own 16 MiB device array."""
    ld = int(X.stride(0)) if ld is None else ld
    _check(lib().consensus_error_noalloc(_ptr(X), n, d, ld, _ptr(out), _ptr(xbar), _stream(stream)))


def ceca_state_consensus(S, n: int, d: int, out, workspace=None, ld: Optional[int] = None, stream=None) -> None:
    """out: device float64 tensor of 11 (x part, y part, ||phi||_F^2); see include/ceca.h."""
    ld = int(S.stride(0)) if ld is None else ld
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().ceca_state_consensus(_ptr(S), n, d, ld, _ptr(out), _ptr(workspace), wbytes, _stream(stream)))


def ceca_stream_probe(a, b, c, o1, o2, count: int, reads: int = 3, writes: int = 2, stream=None) -> None:
    """Measurement aid (ceca_test.h): elementwise kernel with `reads` streaming reads (of a, b, c) and `writes`
    streaming writes (of o1, o2) per element."""
    _check(lib().ceca_stream_probe(_ptr(a), _ptr(b), _ptr(c), _ptr(o1), _ptr(o2), count, reads, writes, _stream(stream)))


def ceca_describe_step_launch(n: int, d: int, ld: int, r: int, port: int, kind: int, in_place: bool) -> dict:
    """Launch shape the library picks for the state-updating kernel of a gossip round (kind 0), a fused
    quadratic-centre step (1) or a minibatch step's combine (2) (ceca_test.h)."""
    out = (C.c_int32 * 6)()
    _check(lib().ceca_describe_step_launch(n, d, ld, r, port, int(kind), int(in_place), out))
    return dict(zip(("rows", "band", "wg_per_cu", "stretch", "stretches_per_cycle", "vec"), list(out)))


def ceca_set_option(option: int, value: int) -> None:
    """Launch-shape override of the calling thread (ceca_test.h)."""
    _check(lib().ceca_set_option(option, value))


def ceca_reset_options() -> None:
    """Every launch-shape override of the calling thread back to the library default (ceca_test.h)."""
    _check(lib().ceca_reset_options())


def make_minibatch_loss(kind: int, A, t, N: int, B: int, grad_scale: float = 0.0, noise_std: float = 0.0,
                        seed: int = 0, k: int = 0) -> Loss:
    """A: device (n, N, lda) float32, t: device (n, N) float32.  grad_scale = 0 means the mean over the batch."""
    return Loss(kind=kind, N=N, B=B, seed=seed & 0xFFFFFFFF, k=k & 0xFFFFFFFF, noise_std=noise_std,
                grad_scale=grad_scale, A=_ptr(A), lda=int(A.stride(-2)), t=_ptr(t), c=None, ldc=0)


def make_quad_center_loss(c, noise_std: float, seed: int, k: int = 0) -> Loss:
    """c: device (n, ldc) float32 centres."""
    return Loss(kind=LOSS_QUAD_CENTER, N=0, B=0, seed=seed & 0xFFFFFFFF, k=k & 0xFFFFFFFF, noise_std=noise_std,
                grad_scale=0.0, A=None, lda=0, t=None, c=_ptr(c), ldc=int(c.stride(0)))


def make_gradient_loss(e) -> Loss:
    """e: device (n, ldc) float32, row i = agent i's stochastic gradient evaluated by the caller at z_i (the x
    row when the round's exchange_y is 0, the y row when it is 1)."""
    return Loss(kind=LOSS_GRADIENT, N=0, B=0, seed=0, k=0, noise_std=0.0, grad_scale=0.0, A=None, lda=0, t=None,
                c=_ptr(e), ldc=int(e.stride(0)))
