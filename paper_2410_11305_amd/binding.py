"""ctypes binding of libqspec.so: same names as the C ABI (include/qspec.h),
argument marshalling only.  Tensors are torch CUDA tensors; torch provides the
device memory and the stream, every computation runs in the HIP library.
There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqspec.so")
GROUP = 128

OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_WORKSPACE, ERR_HIP, ERR_UNSUPPORTED = range(7)

EXPORTS = (
    "qspec_status_string", "qspec_version", "qspec_packed_weight_bytes", "qspec_workspace_bytes",
    "qspec_pack_weights", "qspec_unpack_weights", "qspec_quant_act", "qspec_gemm_w4a4",
    "qspec_gemm_w4a16", "qspec_gemm_w4a4_partials", "qspec_describe_kernel",
    "qspec_accept_workspace_bytes", "qspec_greedy_accept", "qspec_kv_overwrite",
    "qspec_rmsnorm_quant", "qspec_silu_mul_quant", "qspec_hadamard_quant",
    "qspec_reorder_quant", "qspec_debug_set_plan",
    "qspec_gemm_w4a16_noalloc", "qspec_mlp_draft", "qspec_mlp_draft_workspace_bytes",
    "qspec_w4a4_takes_wide", "qspec_quant_act_wide", "qspec_gemm_w4a4_wide",
)


class QSpecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libqspec.so (built by `python -m paper_2410_11305_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2410_11305_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.qspec_status_string.restype = ctypes.c_char_p
    L.qspec_status_string.argtypes = [ci]
    L.qspec_version.restype = ci
    L.qspec_version.argtypes = []
    L.qspec_packed_weight_bytes.restype = sz
    L.qspec_packed_weight_bytes.argtypes = [ci, ci, ci]
    L.qspec_workspace_bytes.restype = sz
    L.qspec_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.qspec_pack_weights.restype = ci
    L.qspec_pack_weights.argtypes = [vp, vp, ci, ci, ci, vp, vp]
    L.qspec_w4a4_takes_wide.restype = ci
    L.qspec_w4a4_takes_wide.argtypes = [ci, ci, ci, ci]
    L.qspec_quant_act_wide.restype = ci
    L.qspec_quant_act_wide.argtypes = [vp, ci, ci, ci, vp, vp, vp]
    L.qspec_gemm_w4a4_wide.restype = ci
    L.qspec_gemm_w4a4_wide.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    L.qspec_unpack_weights.restype = ci
    L.qspec_unpack_weights.argtypes = [vp, ci, ci, ci, vp, vp, vp]
    L.qspec_quant_act.restype = ci
    L.qspec_quant_act.argtypes = [vp, ci, ci, ci, vp, vp, vp]
    L.qspec_gemm_w4a4.restype = ci
    L.qspec_gemm_w4a4.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    L.qspec_gemm_w4a16.restype = ci
    L.qspec_gemm_w4a16.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    L.qspec_gemm_w4a4_partials.restype = ci
    L.qspec_gemm_w4a4_partials.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    L.qspec_describe_kernel.restype = ci
    L.qspec_describe_kernel.argtypes = [ci, ci, ci, ci, ci, ctypes.c_char_p, sz]
    L.qspec_accept_workspace_bytes.restype = sz
    L.qspec_accept_workspace_bytes.argtypes = [ci, ci, ci]
    L.qspec_greedy_accept.restype = ci
    L.qspec_greedy_accept.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, sz, vp]
    L.qspec_kv_overwrite.restype = ci
    L.qspec_kv_overwrite.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
    L.qspec_rmsnorm_quant.restype = ci
    L.qspec_rmsnorm_quant.argtypes = [vp, vp, ctypes.c_float, ci, ci, ci, ci, vp, vp, vp, vp]
    L.qspec_silu_mul_quant.restype = ci
    L.qspec_silu_mul_quant.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp]
    L.qspec_hadamard_quant.restype = ci
    L.qspec_hadamard_quant.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    L.qspec_reorder_quant.restype = ci
    L.qspec_reorder_quant.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp]
    L.qspec_gemm_w4a16_noalloc.restype = ci
    L.qspec_gemm_w4a16_noalloc.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    L.qspec_mlp_draft_workspace_bytes.restype = sz
    L.qspec_mlp_draft_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.qspec_mlp_draft.restype = ci
    L.qspec_mlp_draft.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp, vp]
    L.qspec_debug_set_plan.restype = ci
    L.qspec_debug_set_plan.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().qspec_status_string(int(status)).decode()


def version() -> int:
    return lib().qspec_version()


def packed_weight_bytes(N: int, K: int, group: int = GROUP) -> int:
    return lib().qspec_packed_weight_bytes(N, K, group)


def workspace_bytes(M: int, N: int, K: int, group: int = GROUP) -> int:
    return lib().qspec_workspace_bytes(M, N, K, group)


def debug_set_plan(name: str, value: str = None) -> None:
    """Force (value) or release (None) one of the library's kernel-plan overrides."""
    _check(lib().qspec_debug_set_plan(name.encode(), None if value is None else str(value).encode()),
           "qspec_debug_set_plan")


def describe_kernel(w4a4: bool, M: int, N: int, K: int, group: int = GROUP) -> str:
    buf = ctypes.create_string_buffer(128)
    _check(lib().qspec_describe_kernel(1 if w4a4 else 0, M, N, K, group, buf, 128), "qspec_describe_kernel")
    return buf.value.decode()


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != OK:
        raise QSpecError(status, where)


def alloc_workspace(nbytes: int) -> torch.Tensor:
    """A workspace for the GEMM entry points.  Zero-filled: the head of a workspace
    holds arrival counters that must be zero before its first use (every call
    leaves them zero again, so one workspace serves any number of calls in turn)."""
    return torch.zeros(max(int(nbytes), 16), dtype=torch.uint8, device="cuda")


def _workspace(M, N, K, group, workspace):
    need = workspace_bytes(M, N, K, group)
    if workspace is None:
        if need == 0:
            return None, 0
        # convenience for tests: hot loops pass a workspace from alloc_workspace instead
        workspace = alloc_workspace(need)
    return _dev(workspace, torch.uint8, "workspace"), workspace.numel()


def pack_weights(codes: torch.Tensor, scales: torch.Tensor, packed: torch.Tensor = None,
                 group: int = GROUP) -> torch.Tensor:
    """codes int8 [N,K] in [-8,7], scales fp16 [N,K/128] -> uint8 blob."""
    N, K = codes.shape
    if packed is None:
        nbytes = packed_weight_bytes(N, K, group)
        if nbytes == 0:
            raise QSpecError(ERR_SHAPE, "qspec_pack_weights")
        packed = torch.empty(nbytes, dtype=torch.uint8, device=codes.device)
    _check(lib().qspec_pack_weights(_dev(codes, torch.int8, "codes"), _dev(scales, torch.float16, "scales"),
                                    N, K, group, _dev(packed, torch.uint8, "packed"), _stream()),
           "qspec_pack_weights")
    return packed


def unpack_weights(packed: torch.Tensor, N: int, K: int, group: int = GROUP):
    codes = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    scales = torch.empty((N, K // group), dtype=torch.float16, device=packed.device)
    _check(lib().qspec_unpack_weights(_dev(packed, torch.uint8, "packed"), N, K, group,
                                      codes.data_ptr(), scales.data_ptr(), _stream()),
           "qspec_unpack_weights")
    return codes, scales


def quant_act(x: torch.Tensor, qa: torch.Tensor = None, sa: torch.Tensor = None, group: int = GROUP):
    """x fp16 [M,K] -> (qa uint8 [M,K/2], sa fp32 [M,K/128])."""
    M, K = x.shape
    if qa is None:
        qa = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    if sa is None:
        sa = torch.empty((M, max(K // group, 1)), dtype=torch.float32, device=x.device)
    _check(lib().qspec_quant_act(_dev(x, torch.float16, "x"), M, K, group,
                                 _dev(qa, torch.uint8, "qa"), _dev(sa, torch.float32, "sa"), _stream()),
           "qspec_quant_act")
    return qa, sa


def w4a4_takes_wide(M: int, N: int, K: int, group: int = GROUP) -> bool:
    """True when the draft-mode GEMM of this shape runs on the kernel that can take the widened
    activation format (quant_act_wide -> gemm_w4a4_wide)."""
    return bool(lib().qspec_w4a4_takes_wide(M, N, K, group))


def quant_act_wide(x: torch.Tensor, qa8: torch.Tensor = None, sa: torch.Tensor = None, group: int = GROUP):
    """x fp16 [M,K] -> (qa8 int8 [M,K] in the widened device format, sa fp32 [M,K/128])."""
    M, K = x.shape
    if qa8 is None:
        qa8 = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sa is None:
        sa = torch.empty((M, max(K // group, 1)), dtype=torch.float32, device=x.device)
    _check(lib().qspec_quant_act_wide(_dev(x, torch.float16, "x"), M, K, group,
                                      _dev(qa8, torch.int8, "qa8"), _dev(sa, torch.float32, "sa"), _stream()),
           "qspec_quant_act_wide")
    return qa8, sa


def _quant_outputs(M, K, group, device, qa, sa, h, want_h, wide=False):
    if qa is None:
        qa = (torch.empty((M, K), dtype=torch.int8, device=device) if wide
              else torch.empty((M, K // 2), dtype=torch.uint8, device=device))
    if sa is None:
        sa = torch.empty((M, max(K // group, 1)), dtype=torch.float32, device=device)
    if h is None and want_h:
        h = torch.empty((M, K), dtype=torch.float16, device=device)
    return qa, sa, h


def rmsnorm_quant(x: torch.Tensor, weight: torch.Tensor, eps: float, qa: torch.Tensor = None,
                  sa: torch.Tensor = None, h: torch.Tensor = None, want_h: bool = False, rotate: bool = False,
                  group: int = GROUP, wide: bool = False):
    """RMSNorm (then, if `rotate`, the per-group Hadamard rotation) fused with the activation
    quantiser: x fp16 [M,K], weight fp16 [K] -> (qa uint8 [M,K/2], sa fp32 [M,K/128], h fp16 [M,K] or None);
    `wide`: qa int8 [M,K] in the widened format instead."""
    M, K = x.shape
    qa, sa, h = _quant_outputs(M, K, group, x.device, qa, sa, h, want_h, wide)
    _check(lib().qspec_rmsnorm_quant(_dev(x, torch.float16, "x"), _dev(weight, torch.float16, "weight"),
                                     float(eps), M, K, group, int(bool(rotate)) | (2 if wide else 0),
                                     _dev(qa, torch.int8 if wide else torch.uint8, "qa"),
                                     _dev(sa, torch.float32, "sa"),
                                     None if h is None else _dev(h, torch.float16, "h"), _stream()),
           "qspec_rmsnorm_quant")
    return qa, sa, h


def silu_mul_quant(gate_up: torch.Tensor, qa: torch.Tensor = None, sa: torch.Tensor = None,
                   h: torch.Tensor = None, want_h: bool = False, rotate: bool = False, group: int = GROUP,
                   wide: bool = False):
    """SiLU(gate) * up (then, if `rotate`, the per-group Hadamard rotation) fused with the activation
    quantiser: gate_up fp16 [M,2I] (gate first) -> (qa uint8 [M,I/2], sa fp32 [M,I/128], h fp16 [M,I] or None);
    `wide`: qa int8 [M,I] in the widened format instead."""
    M, I = gate_up.shape[0], gate_up.shape[1] // 2
    qa, sa, h = _quant_outputs(M, I, group, gate_up.device, qa, sa, h, want_h, wide)
    _check(lib().qspec_silu_mul_quant(_dev(gate_up, torch.float16, "gate_up"), M, I, group,
                                      int(bool(rotate)) | (2 if wide else 0),
                                      _dev(qa, torch.int8 if wide else torch.uint8, "qa"), _dev(sa, torch.float32, "sa"),
                                      None if h is None else _dev(h, torch.float16, "h"), _stream()),
           "qspec_silu_mul_quant")
    return qa, sa, h


def hadamard_quant(x: torch.Tensor, qa: torch.Tensor = None, sa: torch.Tensor = None,
                   h: torch.Tensor = None, want_h: bool = False, group: int = GROUP):
    """Every group of 128 features times H_128 / 8, then the activation quantiser: x fp16 [M,K] ->
    (qa uint8 [M,K/2], sa fp32 [M,K/128], h fp16 [M,K] or None)."""
    M, K = x.shape
    qa, sa, h = _quant_outputs(M, K, group, x.device, qa, sa, h, want_h)
    _check(lib().qspec_hadamard_quant(_dev(x, torch.float16, "x"), M, K, group,
                                      _dev(qa, torch.uint8, "qa"), _dev(sa, torch.float32, "sa"),
                                      None if h is None else _dev(h, torch.float16, "h"), _stream()),
           "qspec_hadamard_quant")
    return qa, sa, h


def reorder_quant(x: torch.Tensor, perm: torch.Tensor, n_outlier_groups: int, qa: torch.Tensor = None,
                  sa: torch.Tensor = None, h: torch.Tensor = None, want_h: bool = False, group: int = GROUP):
    """Reordering quantiser: x fp16 [M,K], perm int32 [K] -> (qa uint8 [M,K'/2], sa fp32 [M,K'/128],
    h fp16 [M,K'] or None) with K' = K + 128 * n_outlier_groups."""
    M, K = x.shape
    Kx = K + group * int(n_outlier_groups)
    qa, sa, h = _quant_outputs(M, Kx, group, x.device, qa, sa, h, want_h)
    _check(lib().qspec_reorder_quant(_dev(x, torch.float16, "x"), _dev(perm, torch.int32, "perm"), M, K, group,
                                     int(n_outlier_groups), _dev(qa, torch.uint8, "qa"),
                                     _dev(sa, torch.float32, "sa"),
                                     None if h is None else _dev(h, torch.float16, "h"), _stream()),
           "qspec_reorder_quant")
    return qa, sa, h


def gemm_w4a4(packed: torch.Tensor, qa: torch.Tensor, sa: torch.Tensor, N: int,
              y: torch.Tensor = None, workspace: torch.Tensor = None, group: int = GROUP) -> torch.Tensor:
    M, K = qa.shape[0], qa.shape[1] * 2
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=qa.device)
    ws, ws_bytes = _workspace(M, N, K, group, workspace)
    _check(lib().qspec_gemm_w4a4(_dev(packed, torch.uint8, "packed"), _dev(qa, torch.uint8, "qa"),
                                 _dev(sa, torch.float32, "sa"), M, N, K, group,
                                 _dev(y, torch.float16, "y"), ws, ws_bytes, _stream()),
           "qspec_gemm_w4a4")
    return y


def gemm_w4a4_wide(packed: torch.Tensor, qa8: torch.Tensor, sa: torch.Tensor, N: int,
                   y: torch.Tensor = None, workspace: torch.Tensor = None, group: int = GROUP) -> torch.Tensor:
    M, K = qa8.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=qa8.device)
    ws, ws_bytes = _workspace(M, N, K, group, workspace)
    _check(lib().qspec_gemm_w4a4_wide(_dev(packed, torch.uint8, "packed"), _dev(qa8, torch.int8, "qa8"),
                                      _dev(sa, torch.float32, "sa"), M, N, K, group,
                                      _dev(y, torch.float16, "y"), ws, ws_bytes, _stream()),
           "qspec_gemm_w4a4_wide")
    return y


def gemm_w4a16(packed: torch.Tensor, x: torch.Tensor, N: int, y: torch.Tensor = None,
               workspace: torch.Tensor = None, group: int = GROUP) -> torch.Tensor:
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    ws, ws_bytes = _workspace(M, N, K, group, workspace)
    _check(lib().qspec_gemm_w4a16(_dev(packed, torch.uint8, "packed"), _dev(x, torch.float16, "x"),
                                  M, N, K, group, _dev(y, torch.float16, "y"), ws, ws_bytes, _stream()),
           "qspec_gemm_w4a16")
    return y


NOALLOC_SCRATCH_BYTES = (32 << 20) + 16384


def gemm_w4a16_noalloc(packed: torch.Tensor, x: torch.Tensor, N: int, y: torch.Tensor,
                       group: int = GROUP) -> torch.Tensor:
    """qspec_gemm_w4a16 on the library's built-in scratch: the caller passes every buffer,
    nothing is allocated here or in the library."""
    M, K = x.shape
    _check(lib().qspec_gemm_w4a16_noalloc(_dev(packed, torch.uint8, "packed"), _dev(x, torch.float16, "x"),
                                          M, N, K, group, _dev(y, torch.float16, "y"), _stream()),
           "qspec_gemm_w4a16_noalloc")
    return y


def mlp_draft_workspace_bytes(M: int, H: int, I: int, group: int = GROUP) -> int:
    return lib().qspec_mlp_draft_workspace_bytes(M, H, I, group)


def mlp_draft(packed_gate_up: torch.Tensor, packed_down: torch.Tensor, qa_h: torch.Tensor, sa_h: torch.Tensor,
              H: int, I: int, workspace: torch.Tensor, status: torch.Tensor, gate_up: torch.Tensor = None,
              qa_i: torch.Tensor = None, sa_i: torch.Tensor = None, y: torch.Tensor = None, group: int = GROUP):
    """The draft-pass MLP of a block in one persistent launch.  workspace: zero-filled uint8 of
    mlp_draft_workspace_bytes; status: int32 [1] the caller zeroed (1 afterwards: the launch gave up).
    Returns (gate_up fp16 [M, 2I], qa_i, sa_i, y fp16 [M, H])."""
    M = qa_h.shape[0]
    dev = qa_h.device
    if gate_up is None:
        gate_up = torch.empty((M, 2 * I), dtype=torch.float16, device=dev)
    if qa_i is None:
        qa_i = torch.empty((M, I // 2), dtype=torch.uint8, device=dev)
    if sa_i is None:
        sa_i = torch.empty((M, I // group), dtype=torch.float32, device=dev)
    if y is None:
        y = torch.empty((M, H), dtype=torch.float16, device=dev)
    _check(lib().qspec_mlp_draft(_dev(packed_gate_up, torch.uint8, "packed_gate_up"), _dev(packed_down, torch.uint8, "packed_down"),
                                 _dev(qa_h, torch.uint8, "qa_h"), _dev(sa_h, torch.float32, "sa_h"), M, H, I, group,
                                 _dev(gate_up, torch.float16, "gate_up"), _dev(qa_i, torch.uint8, "qa_i"),
                                 _dev(sa_i, torch.float32, "sa_i"), _dev(y, torch.float16, "y"),
                                 _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                 _dev(status, torch.int32, "status"), _stream()),
           "qspec_mlp_draft")
    return gate_up, qa_i, sa_i, y


def gemm_w4a4_partials(packed: torch.Tensor, qa: torch.Tensor, N: int, n0: int, n_count: int,
                       partials: torch.Tensor = None, group: int = GROUP) -> torch.Tensor:
    M, K = qa.shape[0], qa.shape[1] * 2
    if partials is None:
        partials = torch.empty((M, n_count, K // group), dtype=torch.int32, device=qa.device)
    _check(lib().qspec_gemm_w4a4_partials(_dev(packed, torch.uint8, "packed"), _dev(qa, torch.uint8, "qa"),
                                          M, N, K, group, n0, n_count,
                                          _dev(partials, torch.int32, "partials"), _stream()),
           "qspec_gemm_w4a4_partials")
    return partials


def accept_workspace_bytes(B: int, gamma: int, V: int) -> int:
    return lib().qspec_accept_workspace_bytes(B, gamma, V)


def greedy_accept(logits: torch.Tensor, draft: torch.Tensor, n_accept: torch.Tensor = None,
                  out_tokens: torch.Tensor = None, workspace: torch.Tensor = None):
    """logits fp16 [B, gamma+1, V], draft int32 [B, gamma] -> (n_accept int32 [B], out_tokens int32 [B, gamma+1])."""
    B, rows, V = logits.shape
    gamma = rows - 1
    if n_accept is None:
        n_accept = torch.empty((B,), dtype=torch.int32, device=logits.device)
    if out_tokens is None:
        out_tokens = torch.empty((B, rows), dtype=torch.int32, device=logits.device)
    if workspace is None:
        workspace = torch.empty(max(accept_workspace_bytes(B, gamma, V), 16), dtype=torch.uint8, device=logits.device)
    _check(lib().qspec_greedy_accept(_dev(logits, torch.float16, "logits"), _dev(draft, torch.int32, "draft"),
                                     B, gamma, V, _dev(n_accept, torch.int32, "n_accept"),
                                     _dev(out_tokens, torch.int32, "out_tokens"),
                                     _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()),
           "qspec_greedy_accept")
    return n_accept, out_tokens


def kv_overwrite(cache: torch.Tensor, kv_verify: torch.Tensor, n_accept: torch.Tensor, pos: torch.Tensor) -> torch.Tensor:
    """cache fp16 [B, S, D] (updated in place), kv_verify fp16 [B, gamma+1, D], n_accept / pos int32 [B]."""
    B, S, D = cache.shape
    gamma = kv_verify.shape[1] - 1
    _check(lib().qspec_kv_overwrite(_dev(kv_verify, torch.float16, "kv_verify"), _dev(n_accept, torch.int32, "n_accept"),
                                    _dev(pos, torch.int32, "pos"), B, gamma, D, S,
                                    _dev(cache, torch.float16, "cache"), _stream()),
           "qspec_kv_overwrite")
    return cache
