"""ctypes binding of libcerberus.so: the same entry points as include/cerberus.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of the path runs in
the library's HIP kernels.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch


_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcerberus.so")

CERBERUS_F32, CERBERUS_BF16 = 0, 1
CERBERUS_DEV_KV_OVERFLOW, CERBERUS_DEV_BAD_TOKEN, CERBERUS_DEV_LOG_FULL = 1, 2, 4   # bits of the device status word
CERBERUS_MAX_TREE, CERBERUS_MAX_HEADS, CERBERUS_MAX_TOPK, CERBERUS_MAX_BATCH = 192, 8, 16, 16
DEV_KV_OVERFLOW, DEV_BAD_TOKEN = 1, 2

c_i32p = C.POINTER(C.c_int32)
c_f32p = C.POINTER(C.c_float)
c_vpp = C.POINTER(C.c_void_p)


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "n_cerb_heads", "n_resblocks",
        "special_block", "dtype", "max_batch", "kv_capacity", "topk")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("entropy_threshold", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", c_vpp), ("wqkv", c_vpp), ("wo", c_vpp), ("ffn_norm", c_vpp),
                ("w_gate_up", c_vpp), ("w_down", c_vpp), ("res_w", c_vpp), ("res_b", c_vpp),
                ("head_fc", c_vpp)]


class Tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", c_i32p), ("rank", c_i32p)]


class State(C.Structure):
    _fields_ = [("kv", C.c_void_p), ("kv_len", C.c_void_p), ("root_token", C.c_void_p), ("cand", C.c_void_p),
                ("gate_flag", C.c_void_p), ("entropy", C.c_void_p), ("accept_len", C.c_void_p),
                ("accepted_tokens", C.c_void_p), ("accepted_nodes", C.c_void_p), ("status", C.c_void_p)]


class Taps(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("h_last", C.c_void_p), ("head_logits", C.c_void_p),
                ("node_token", C.c_void_p), ("node_argmax", C.c_void_p), ("forced_node_argmax", C.c_void_p),
                ("forced_gate_hidden", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(or python paper_2410_13344_amd/build.py) first; there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        L.cerberus_workspace_bytes.restype = C.c_size_t
        L.cerberus_workspace_bytes.argtypes = [C.POINTER(Config), C.POINTER(Tree)]
        L.cerberus_init.restype = C.c_int
        L.cerberus_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Config), C.POINTER(Weights), C.POINTER(Tree),
                                    C.c_void_p, C.c_size_t]
        for name in ("cerberus_verify_step", "cerberus_ar_step"):
            f = getattr(L, name)
            f.restype = C.c_int
            f.argtypes = [C.c_void_p, C.POINTER(State), C.c_int32, C.c_void_p]
        L.cerberus_prefill.restype = C.c_int
        L.cerberus_prefill.argtypes = [C.c_void_p, C.POINTER(State), C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        L.cerberus_decode.restype = C.c_int
        L.cerberus_decode.argtypes = [C.c_void_p, C.POINTER(State), C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p]
        L.cerberus_gate.restype = C.c_int
        L.cerberus_gate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.cerberus_accept.restype = C.c_int
        L.cerberus_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(State), C.c_int32, C.c_void_p]
        L.cerberus_accept_noalloc.restype = C.c_int
        L.cerberus_accept_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(State), C.c_int32, C.c_void_p]
        L.cerberus_set_taps.restype = C.c_int
        L.cerberus_set_taps.argtypes = [C.c_void_p, C.POINTER(Taps)]
        L.cerberus_set_param.restype = C.c_int
        L.cerberus_set_param.argtypes = [C.c_void_p, C.c_char_p, C.c_int32]
        L.cerberus_bench_gemm.restype = C.c_int
        L.cerberus_bench_gemm.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.cerberus_last_error.restype = C.c_char_p
        L.cerberus_last_error.argtypes = []
        L.cerberus_destroy.restype = None
        L.cerberus_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


class CerberusError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"cerberus status {code}: {lib().cerberus_last_error().decode()}")


def _check(rc: int) -> None:
    if rc != 0:
        raise CerberusError(rc)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def make_config(cfg: dict, dtype: int, max_batch: int, kv_capacity: int) -> Config:
    return Config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"],
                  cfg["n_cerb_heads"], cfg["n_resblocks"], cfg["special_block"], dtype, max_batch, kv_capacity,
                  cfg["topk"], cfg["rms_eps"], cfg["rope_theta"], cfg["entropy_threshold"])


def make_tree(parent: Sequence[int], rank: Sequence[int]):
    n = len(parent)
    p = (C.c_int32 * n)(*parent)
    r = (C.c_int32 * n)(*rank)
    return Tree(n, C.cast(p, c_i32p), C.cast(r, c_i32p)), (p, r)


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return C.cast(arr, c_vpp), arr


def make_weights(W: dict):
    """W: the dict of device tensors produced by synth.make_weights.  Returns (struct, keepalive)."""
    keep = []

    def arr(ts):
        p, a = _ptr_array(ts)
        keep.append(a)
        keep.append(ts)
        return p

    L = W["layers"]
    res_w = [b["w"] for h in W["heads"] for b in h["blocks"]]
    res_b = [b["b"] for h in W["heads"] for b in h["blocks"]]
    ws = Weights(W["embed"].data_ptr(), W["final_norm"].data_ptr(), W["lm_head"].data_ptr(),
                 arr([l["attn_norm"] for l in L]), arr([l["wqkv"] for l in L]), arr([l["wo"] for l in L]),
                 arr([l["ffn_norm"] for l in L]), arr([l["w_gate_up"] for l in L]), arr([l["w_down"] for l in L]),
                 arr(res_w), arr(res_b), arr([h["fc"] for h in W["heads"]]))
    return ws, keep


# ------------------------------------------------------------------------------------------------
# the entry points, named as in the header
# ------------------------------------------------------------------------------------------------

def cerberus_workspace_bytes(cfg: Config, tree: Tree) -> int:
    return int(lib().cerberus_workspace_bytes(C.byref(cfg), C.byref(tree)))


def cerberus_init(cfg: Config, weights: Weights, tree: Tree, workspace: torch.Tensor) -> int:
    ctx = C.c_void_p()
    _check(lib().cerberus_init(C.byref(ctx), C.byref(cfg), C.byref(weights), C.byref(tree), workspace.data_ptr(),
                               workspace.numel() * workspace.element_size()))
    return ctx.value


def cerberus_verify_step(ctx: int, state: State, batch: int, stream=None) -> None:
    _check(lib().cerberus_verify_step(ctx, C.byref(state), batch, _stream_ptr(stream)))


def cerberus_ar_step(ctx: int, state: State, batch: int, stream=None) -> None:
    _check(lib().cerberus_ar_step(ctx, C.byref(state), batch, _stream_ptr(stream)))


def cerberus_prefill(ctx: int, state: State, batch: int, seq: int, tokens: torch.Tensor, stream=None) -> None:
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.dim() == 1
    _check(lib().cerberus_prefill(ctx, C.byref(state), batch, seq, tokens.data_ptr(), tokens.shape[0], _stream_ptr(stream)))


def cerberus_decode(ctx: int, state: State, batch: int, n_steps: int, out_tokens: torch.Tensor, out_count: torch.Tensor,
                    stream=None) -> None:
    _check(lib().cerberus_decode(ctx, C.byref(state), batch, n_steps, out_tokens.data_ptr(), out_tokens.shape[1],
                                 out_count.data_ptr(), _stream_ptr(stream)))


def cerberus_gate(ctx: int, hidden: torch.Tensor, entropy_out: torch.Tensor, flag_out: torch.Tensor, stream=None) -> None:
    _check(lib().cerberus_gate(ctx, hidden.data_ptr(), hidden.shape[0], entropy_out.data_ptr(), flag_out.data_ptr(),
                               _stream_ptr(stream)))


def cerberus_accept(ctx: int, node_argmax: torch.Tensor, node_token: torch.Tensor, state: State, batch: int,
                    stream=None) -> None:
    _check(lib().cerberus_accept(ctx, node_argmax.data_ptr(), node_token.data_ptr(), C.byref(state), batch,
                                 _stream_ptr(stream)))


def cerberus_accept_noalloc(ctx: int, node_argmax: torch.Tensor, node_token: torch.Tensor, state: State, batch: int,
                            stream=None) -> None:
    _check(lib().cerberus_accept_noalloc(ctx, node_argmax.data_ptr(), node_token.data_ptr(), C.byref(state), batch,
                                         _stream_ptr(stream)))


def cerberus_set_taps(ctx: int, taps: Optional[Taps]) -> None:
    _check(lib().cerberus_set_taps(ctx, C.byref(taps) if taps is not None else None))


def cerberus_set_param(ctx: int, name: str, value: int) -> None:
    _check(lib().cerberus_set_param(ctx, name.encode(), value))


def cerberus_bench_gemm(ctx: int, kind: int, rows: int, stream=None) -> float:
    nbytes = C.c_double(0.0)
    _check(lib().cerberus_bench_gemm(ctx, kind, rows, _stream_ptr(stream), C.byref(nbytes)))
    return nbytes.value


def cerberus_destroy(ctx: int) -> None:
    lib().cerberus_destroy(ctx)


# ------------------------------------------------------------------------------------------------
# allocation helpers (device memory comes from torch)
# ------------------------------------------------------------------------------------------------

class DeviceState:
    """Owns the device arrays of a cerberus_state for `max_batch` sequences."""

    def __init__(self, cfg: dict, dtype: int, max_batch: int, kv_capacity: int, device="cuda"):
        tdt = torch.float32 if dtype == CERBERUS_F32 else torch.bfloat16
        Hc, K = cfg["n_cerb_heads"], cfg["topk"]
        i32 = dict(dtype=torch.int32, device=device)
        self.kv = torch.zeros((cfg["n_layers"], 2, max_batch, cfg["n_heads"], kv_capacity, cfg["head_dim"]),
                              dtype=tdt, device=device)
        self.kv_len = torch.zeros(max_batch, **i32)
        self.root_token = torch.zeros(max_batch, **i32)
        self.cand = torch.zeros((max_batch, Hc, K), **i32)
        self.gate_flag = torch.zeros(max_batch, **i32)
        self.entropy = torch.zeros(max_batch, dtype=torch.float32, device=device)
        self.accept_len = torch.zeros(max_batch, **i32)
        self.accepted_tokens = torch.zeros((max_batch, Hc + 1), **i32)
        self.accepted_nodes = torch.zeros((max_batch, Hc + 1), **i32)
        self.status = torch.zeros(1, **i32)
        self.struct = State(*[getattr(self, n).data_ptr() for n, _ in State._fields_])


class DeviceTaps:
    def __init__(self, cfg: dict, max_batch: int, T: int, device="cuda", logits=True, forced_argmax=False,
                 forced_gate=False):
        f32 = dict(dtype=torch.float32, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        R = max_batch * T
        self.logits = torch.zeros((R, cfg["vocab"]), **f32) if logits else None
        self.h_last = torch.zeros((R, cfg["d_model"]), **f32)
        self.head_logits = torch.zeros((max_batch, cfg["n_cerb_heads"], cfg["vocab"]), **f32)
        self.node_token = torch.zeros(R, **i32)
        self.node_argmax = torch.zeros(R, **i32)
        self.forced_node_argmax = torch.zeros(R, **i32) if forced_argmax else None
        self.forced_gate_hidden = torch.zeros((max_batch, cfg["d_model"]), **f32) if forced_gate else None
        self.struct = Taps(*[_ptr(getattr(self, n)) for n, _ in Taps._fields_])


class Engine:
    """A context plus the buffers that must outlive it."""

    def __init__(self, cfg: dict, W: dict, parent, rank, dtype: int, max_batch: int, kv_capacity: int):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the Cerberus library only runs on a HIP device")
        self.cfg, self.dtype, self.max_batch, self.kv_capacity = cfg, dtype, max_batch, kv_capacity
        self.T = len(parent)
        self.c_cfg = make_config(cfg, dtype, max_batch, kv_capacity)
        self.c_tree, self._tree_keep = make_tree(parent, rank)
        self.c_weights, self._w_keep = make_weights(W)
        nbytes = cerberus_workspace_bytes(self.c_cfg, self.c_tree)
        if nbytes == 0:
            raise CerberusError(-2)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.ctx = cerberus_init(self.c_cfg, self.c_weights, self.c_tree, self.workspace)

    def new_state(self) -> DeviceState:
        return DeviceState(self.cfg, self.dtype, self.max_batch, self.kv_capacity)

    def verify_step(self, st: DeviceState, batch: int, stream=None):
        cerberus_verify_step(self.ctx, st.struct, batch, stream)

    def ar_step(self, st: DeviceState, batch: int, stream=None):
        cerberus_ar_step(self.ctx, st.struct, batch, stream)

    def prefill(self, st: DeviceState, batch: int, seq: int, tokens: torch.Tensor, stream=None):
        cerberus_prefill(self.ctx, st.struct, batch, seq, tokens, stream)

    def decode(self, st: DeviceState, batch: int, n_steps: int, out_tokens: torch.Tensor, out_count: torch.Tensor,
               stream=None):
        cerberus_decode(self.ctx, st.struct, batch, n_steps, out_tokens, out_count, stream)

    def generate(self, st: DeviceState, prompts, n_steps: int, stream=None):
        """Prompt phase for every sequence, then n_steps chained decoding steps (Algorithm 1 from its
        first line to its last); returns the committed token ids of every sequence.  Only calls and
        buffers: everything is computed by cerberus_prefill and cerberus_decode."""
        batch = len(prompts)
        st.kv_len[:batch] = 0
        for b, p in enumerate(prompts):
            self.prefill(st, batch, b, p.to(device="cuda", dtype=torch.int32), stream)
        cap = n_steps * (self.cfg["n_cerb_heads"] + 1)
        log = torch.full((batch, cap), -1, dtype=torch.int32, device="cuda")
        count = torch.zeros(batch, dtype=torch.int32, device="cuda")
        self.decode(st, batch, n_steps, log, count, stream)
        torch.cuda.synchronize()
        return [log[b, :int(count[b])].cpu().tolist() for b in range(batch)]

    def set_taps(self, taps: Optional[DeviceTaps]):
        self._taps = taps
        cerberus_set_taps(self.ctx, taps.struct if taps is not None else None)

    def set_param(self, name: str, value: int):
        cerberus_set_param(self.ctx, name, value)

    def close(self):
        if self.ctx:
            cerberus_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
