"""MI355X-native hot path of Alignment-Augmented Speculative Decoding (AASD).

Thin Python binding over the C ABI in ``include/aasd.h``: argument marshalling only.
Every step of the path (alignment sampling, n-gram draft retrieval, conditional
verification) runs in the hand-written HIP kernels of ``libaasd.so``; PyTorch is used
for device memory and streams, nothing else.  There is no CPU fallback.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import _lib

F32, BF16 = 0, 1
EXTRAS_TOP, EXTRAS_SAMPLE, EXTRAS_GUMBEL = 0, 1, 2
VERIFY_NO_CLAMP = 1
VERIFY_ZEROED_WORKSPACE = 2

MAX_EXTRAS, MAX_CANDSET, MAX_KEY, MAX_DRAFT, MAX_CANDIDATES = 4, 8, 8, 16, 32
MAX_TREE_NODES = 512
HASH_BASE = 0x9E3779B1  # multiplier of the retrieval kernel's window hash (mod 2^32)


class AasdError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"aasd error {code}: {message}")
        self.code = code


def version() -> str:
    return _lib.load().aasd_version().decode()


def _check(rc: int):
    if rc != 0:
        raise AasdError(rc, _lib.load().aasd_last_error().decode())


def set_sweep_events(start, stop):
    """Measurement hook: raw hipEvent_t handles (ints) recorded around the row-sweep kernel; None, None = off."""
    _lib.load().aasd_hook_sweep_events(start, stop)


def set_draw_events(start, stop):
    """The same hook around the kernel that makes the full-vocabulary draws of EXTRAS_GUMBEL."""
    _lib.load().aasd_hook_draw_events(start, stop)


def set_sweep_plan(threads: int = 0, loads: int = 0, segments: int = 0):
    """Test hook: force the launch shape of the row sweep for this thread; (0, 0, 0) = the library picks."""
    _check(_lib.load().aasd_hook_sweep_plan(threads, loads, segments))


def verify_launches(B: int, C: int, k: int, V: int, dt: int, zeroed_workspace: bool = False) -> int:
    """Measurement hook: the number of kernels aasd_verify would enqueue for these sizes (1 = the one-launch form)."""
    return int(_lib.load().aasd_hook_verify_launches(B, C, k, V, dt, VERIFY_ZEROED_WORKSPACE if zeroed_workspace else 0))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def _dev_check(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live on the GPU")


def align_sample(logits: torch.Tensor, next_tok: Optional[torch.Tensor], m: int = 2, c: int = 4,
                 mode: int = EXTRAS_TOP, seed: int = 0, row_id_base: int = 0, V: Optional[int] = None,
                 want_rank: bool = True, near_count: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None):
    """aasd_align_sample over logits[rows, row_stride] (fp32 or bf16, rows contiguous in memory).

    Returns a dict of device tensors: argmax, misaligned, entropy, p_next, p_max, rank (or None),
    extras [rows, m], n_extras.  ``out`` may carry preallocated tensors of the same names."""
    _dev_check(logits, next_tok, near_count)
    assert logits.dim() == 2 and logits.stride(1) == 1
    rows, row_stride = logits.shape[0], logits.stride(0) if logits.shape[0] > 1 else logits.shape[1]
    V = logits.shape[1] if V is None else V
    dev = logits.device
    if out is None:
        out = {}
    o = dict(
        argmax=out.get("argmax", None), misaligned=out.get("misaligned", None), entropy=out.get("entropy", None),
        workspace=None,
        p_next=out.get("p_next", None), p_max=out.get("p_max", None), rank=out.get("rank", None),
        extras=out.get("extras", None), n_extras=out.get("n_extras", None))
    if o["argmax"] is None: o["argmax"] = torch.empty(rows, dtype=torch.int32, device=dev)
    if o["misaligned"] is None: o["misaligned"] = torch.empty(rows, dtype=torch.uint8, device=dev)
    if o["entropy"] is None: o["entropy"] = torch.empty(rows, dtype=torch.float32, device=dev)
    if o["p_next"] is None: o["p_next"] = torch.empty(rows, dtype=torch.float32, device=dev)
    if o["p_max"] is None: o["p_max"] = torch.empty(rows, dtype=torch.float32, device=dev)
    if o["rank"] is None and want_rank: o["rank"] = torch.empty(rows, dtype=torch.int32, device=dev)
    if o["extras"] is None: o["extras"] = torch.empty((rows, m), dtype=torch.int32, device=dev)
    if o["n_extras"] is None: o["n_extras"] = torch.empty(rows, dtype=torch.uint8, device=dev)
    if next_tok is not None:
        assert next_tok.dtype == torch.int32 and next_tok.is_contiguous() and next_tok.numel() == rows
    ws_bytes = align_sample_workspace_bytes(rows, V, _dtype_code(logits))
    if workspace is None:
        workspace = out.get("workspace")
    if workspace is None or workspace.numel() * workspace.element_size() < ws_bytes:
        workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    o["workspace"] = workspace
    rc = _lib.load().aasd_align_sample(
        logits.data_ptr(), _dtype_code(logits), rows, V, row_stride, _ptr(next_tok), m, c, mode,
        seed & 0xFFFFFFFFFFFFFFFF, row_id_base & 0xFFFFFFFFFFFFFFFF,
        o["argmax"].data_ptr(), o["misaligned"].data_ptr(), o["entropy"].data_ptr(), o["p_next"].data_ptr(),
        o["p_max"].data_ptr(), _ptr(o["rank"]), o["extras"].data_ptr(), o["n_extras"].data_ptr(),
        _ptr(near_count), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(dev))
    _check(rc)
    return o


def align_sample_workspace_bytes(rows: int, V: int, dt: int) -> int:
    return int(_lib.load().aasd_align_sample_workspace_bytes(rows, V, dt))


def retrieve_drafts(tokens: torch.Tensor, length: torch.Tensor, prompt_len: torch.Tensor, n_min: int, n_max: int,
                    k: int, C: int, extras: Optional[torch.Tensor] = None, n_extras: Optional[torch.Tensor] = None,
                    m: int = 0, extras_stride: int = 0, want_draft_extras: Optional[bool] = None,
                    out: Optional[dict] = None):
    """aasd_retrieve_drafts over tokens[B, tok_stride] (int32).  Returns a dict of device tensors:
    drafts [B,C,k], draft_len [B,C], src_pos [B,C], n_cand [B], key_len [B], strict [B,C,k],
    draft_extras [B,C,k,m] or None."""
    _dev_check(tokens, length, prompt_len, extras, n_extras)
    assert tokens.dim() == 2 and tokens.dtype == torch.int32 and tokens.stride(1) == 1
    B = tokens.shape[0]
    tok_stride = tokens.stride(0) if B > 1 else tokens.shape[1]
    assert length.dtype == torch.int32 and prompt_len.dtype == torch.int32
    dev = tokens.device
    have_table = extras is not None
    if want_draft_extras is None:
        want_draft_extras = have_table
    if out is None:
        out = {}
    o = dict(out)
    def need(name, shape, dtype):
        if o.get(name) is None:
            o[name] = torch.empty(shape, dtype=dtype, device=dev)
    need("drafts", (B, C, k), torch.int32)
    need("draft_len", (B, C), torch.int32)
    need("src_pos", (B, C), torch.int32)
    need("n_cand", (B,), torch.int32)
    need("key_len", (B,), torch.int32)
    need("strict", (B, C, k), torch.uint8)
    if want_draft_extras:
        need("draft_extras", (B, C, k, m), torch.int32)
    else:
        o["draft_extras"] = None
    rc = _lib.load().aasd_retrieve_drafts(
        tokens.data_ptr(), tok_stride, length.data_ptr(), prompt_len.data_ptr(), B, n_min, n_max, k, C,
        _ptr(extras), _ptr(n_extras), m, extras_stride,
        o["drafts"].data_ptr(), o["draft_len"].data_ptr(), o["src_pos"].data_ptr(), o["n_cand"].data_ptr(),
        o["key_len"].data_ptr(), _ptr(o["draft_extras"]), o["strict"].data_ptr(), _stream(dev))
    _check(rc)
    return o


class DraftPool:
    """Persistent draft pool (aasd_pool_*): device memory plus the parameters that every call repeats."""

    def __init__(self, B: int, capacity: int, n_min: int, n_max: int, device):
        self.B, self.capacity, self.n_min, self.n_max = B, capacity, n_min, n_max
        nbytes = int(_lib.load().aasd_pool_bytes(B, capacity, n_min, n_max))
        if nbytes == 0 and B > 0:
            raise ValueError("invalid pool parameters")
        self.mem = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)

    @property
    def nbytes(self) -> int:
        return self.mem.numel()

    def update(self, tokens: torch.Tensor, length: torch.Tensor, reset: bool = False):
        """Index tokens[b, :length[b]]: everything (reset) or the positions added since the last call."""
        _dev_check(tokens, length)
        assert tokens.dim() == 2 and tokens.dtype == torch.int32 and tokens.stride(1) == 1 and tokens.shape[0] == self.B
        assert length.dtype == torch.int32 and length.shape == (self.B,)
        tok_stride = tokens.stride(0) if self.B > 1 else tokens.shape[1]
        rc = _lib.load().aasd_pool_update(self.mem.data_ptr(), self.nbytes, self.B, self.capacity, self.n_min, self.n_max,
                                          tokens.data_ptr(), tok_stride, length.data_ptr(), 1 if reset else 0,
                                          _stream(tokens.device))
        _check(rc)

    def step(self, *args, **kw):
        """aasd_pool_step: index the tokens added since the last call, then look up (one launch)."""
        return self.retrieve(*args, _update_first=True, **kw)

    def retrieve(self, tokens: torch.Tensor, length: torch.Tensor, prompt_len: torch.Tensor, k: int, C: int,
                 extras: Optional[torch.Tensor] = None, n_extras: Optional[torch.Tensor] = None, m: int = 0,
                 extras_stride: int = 0, want_draft_extras: Optional[bool] = None, out: Optional[dict] = None,
                 _update_first: bool = False):
        """aasd_pool_retrieve: the outputs of retrieve_drafts, found through the pool."""
        _dev_check(tokens, length, prompt_len, extras, n_extras)
        assert tokens.dim() == 2 and tokens.dtype == torch.int32 and tokens.stride(1) == 1 and tokens.shape[0] == self.B
        B = self.B
        tok_stride = tokens.stride(0) if B > 1 else tokens.shape[1]
        assert length.dtype == torch.int32 and prompt_len.dtype == torch.int32
        dev = tokens.device
        have_table = extras is not None
        if want_draft_extras is None:
            want_draft_extras = have_table
        o = dict(out or {})
        def need(name, shape, dtype):
            if o.get(name) is None:
                o[name] = torch.empty(shape, dtype=dtype, device=dev)
        need("drafts", (B, C, k), torch.int32)
        need("draft_len", (B, C), torch.int32)
        need("src_pos", (B, C), torch.int32)
        need("n_cand", (B,), torch.int32)
        need("key_len", (B,), torch.int32)
        need("strict", (B, C, k), torch.uint8)
        if want_draft_extras:
            need("draft_extras", (B, C, k, m), torch.int32)
        else:
            o["draft_extras"] = None
        fn = _lib.load().aasd_pool_step if _update_first else _lib.load().aasd_pool_retrieve
        rc = fn(
            self.mem.data_ptr(), self.nbytes, B, self.capacity, self.n_min, self.n_max,
            tokens.data_ptr(), tok_stride, length.data_ptr(), prompt_len.data_ptr(), k, C,
            _ptr(extras), _ptr(n_extras), m, extras_stride,
            o["drafts"].data_ptr(), o["draft_len"].data_ptr(), o["src_pos"].data_ptr(), o["n_cand"].data_ptr(),
            o["key_len"].data_ptr(), _ptr(o["draft_extras"]), o["strict"].data_ptr(), _stream(dev))
        _check(rc)
        return o


def verify_workspace_bytes(B: int, C: int, k: int, V: int, dt: int) -> int:
    return int(_lib.load().aasd_verify_workspace_bytes(B, C, k, V, dt))


def verify(logits: torch.Tensor, drafts: torch.Tensor, draft_len: torch.Tensor, strict: Optional[torch.Tensor] = None,
           alpha: float = 0.1, beta: float = 0.1, flags: int = 0, V: Optional[int] = None,
           want_rows: bool = True, want_tokens: bool = True, want_near: bool = True,
           workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None, zeroed_workspace: bool = False):
    """aasd_verify over logits[B, R, row_stride], R = 1 + C*k, drafts [B,C,k], draft_len [B,C].

    Returns a dict of device tensors: accept_len, best_cand, next_token [B]; row_entropy, row_pmax,
    row_argmax [B,R]; tok_p, tok_delta [B,C,k]; near_count [B] (the optional ones may be None).
    zeroed_workspace=True passes AASD_VERIFY_ZEROED_WORKSPACE (one launch): the workspace given must have been
    zero-filled once and used since only by such calls with the same B."""
    _dev_check(logits, drafts, draft_len, strict, workspace)
    assert logits.dim() == 3 and logits.stride(2) == 1
    B, R = logits.shape[0], logits.shape[1]
    assert drafts.dtype == torch.int32 and drafts.is_contiguous() and draft_len.dtype == torch.int32
    _, C, k = drafts.shape
    assert R == 1 + C * k, (R, C, k)
    row_stride = logits.stride(1)
    seq_stride = logits.stride(0) if B > 1 else R * row_stride
    V = logits.shape[2] if V is None else V
    dev = logits.device
    if out is None:
        out = {}
    o = dict(out)
    def need(name, shape, dtype, wanted=True):
        if not wanted:
            o[name] = None
        elif o.get(name) is None:
            o[name] = torch.empty(shape, dtype=dtype, device=dev)
    need("accept_len", (B,), torch.int32)
    need("best_cand", (B,), torch.int32)
    need("next_token", (B,), torch.int32)
    need("row_entropy", (B, R), torch.float32, want_rows)
    need("row_pmax", (B, R), torch.float32, want_rows)
    need("row_argmax", (B, R), torch.int32, want_rows)
    need("tok_p", (B, C, k), torch.float32, want_tokens)
    need("tok_delta", (B, C, k), torch.float32, want_tokens)
    need("near_count", (B,), torch.int32, want_near)
    ws_bytes = verify_workspace_bytes(B, C, k, V, _dtype_code(logits))
    if workspace is None:
        workspace = o.get("workspace")
    if workspace is None or workspace.numel() * workspace.element_size() < ws_bytes:
        if zeroed_workspace:
            raise ValueError("zeroed_workspace=True needs the caller's own zero-filled workspace of sufficient size")
        workspace = torch.empty(max(ws_bytes, 32), dtype=torch.uint8, device=dev)
    if zeroed_workspace:
        flags |= VERIFY_ZEROED_WORKSPACE
    rc = _lib.load().aasd_verify(
        logits.data_ptr(), _dtype_code(logits), B, C, k, V, row_stride, seq_stride,
        drafts.data_ptr(), draft_len.data_ptr(), _ptr(strict), float(alpha), float(beta), flags,
        o["accept_len"].data_ptr(), o["best_cand"].data_ptr(), o["next_token"].data_ptr(),
        _ptr(o["row_entropy"]), _ptr(o["row_pmax"]), _ptr(o["row_argmax"]), _ptr(o["tok_p"]), _ptr(o["tok_delta"]),
        _ptr(o["near_count"]), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(dev))
    _check(rc)
    o["workspace"] = workspace
    return o


def verify_static(logits: torch.Tensor, drafts: torch.Tensor, draft_len: torch.Tensor, strict: Optional[torch.Tensor],
                  out: dict, alpha: float = 0.1, beta: float = 0.1, flags: int = 0, V: Optional[int] = None):
    """aasd_verify_static: aasd_verify on the library's built-in scratch memory.  Nothing is allocated, here
    or in the library: `out` must carry accept_len, best_cand, next_token [B] (int32) and may carry row_entropy,
    row_pmax, row_argmax [B,R], tok_p, tok_delta [B,C,k], near_count [B]; it is returned."""
    B, R = logits.shape[0], logits.shape[1]
    _, C, k = drafts.shape
    row_stride = logits.stride(1)
    seq_stride = logits.stride(0) if B > 1 else R * row_stride
    V = logits.shape[2] if V is None else V
    rc = _lib.load().aasd_verify_static(
        logits.data_ptr(), _dtype_code(logits), B, C, k, V, row_stride, seq_stride,
        drafts.data_ptr(), draft_len.data_ptr(), _ptr(strict), float(alpha), float(beta), flags,
        out["accept_len"].data_ptr(), out["best_cand"].data_ptr(), out["next_token"].data_ptr(),
        _ptr(out.get("row_entropy")), _ptr(out.get("row_pmax")), _ptr(out.get("row_argmax")), _ptr(out.get("tok_p")),
        _ptr(out.get("tok_delta")), _ptr(out.get("near_count")), _stream(logits.device))
    _check(rc)
    return out


def verify_static_max_bytes() -> int:
    return int(_lib.load().aasd_verify_static_max_bytes())


def verify_topk_workspace_bytes(B: int, C: int, k: int, V: int, dt: int) -> int:
    return int(_lib.load().aasd_verify_topk_workspace_bytes(B, C, k, V, dt))


def verify_topk(logits: torch.Tensor, drafts: torch.Tensor, draft_len: torch.Tensor, topk: int = 5,
                V: Optional[int] = None, want_rows: bool = True, want_tokens: bool = True,
                workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None):
    """aasd_verify_topk over logits[B, R, row_stride], R = 1 + C*k, drafts [B,C,k], draft_len [B,C].

    Returns a dict of device tensors: accept_len, best_cand, next_token [B]; row_argmax [B,R]; tok_pass [B,C,k]."""
    _dev_check(logits, drafts, draft_len, workspace)
    assert logits.dim() == 3 and logits.stride(2) == 1
    B, R = logits.shape[0], logits.shape[1]
    assert drafts.dtype == torch.int32 and drafts.is_contiguous() and draft_len.dtype == torch.int32
    _, C, k = drafts.shape
    assert R == 1 + C * k, (R, C, k)
    row_stride = logits.stride(1)
    seq_stride = logits.stride(0) if B > 1 else R * row_stride
    V = logits.shape[2] if V is None else V
    dev = logits.device
    o = dict(out or {})
    def need(name, shape, dtype, wanted=True):
        if not wanted:
            o[name] = None
        elif o.get(name) is None:
            o[name] = torch.empty(shape, dtype=dtype, device=dev)
    need("accept_len", (B,), torch.int32)
    need("best_cand", (B,), torch.int32)
    need("next_token", (B,), torch.int32)
    need("row_argmax", (B, R), torch.int32, want_rows)
    need("tok_pass", (B, C, k), torch.uint8, want_tokens)
    ws_bytes = verify_topk_workspace_bytes(B, C, k, V, _dtype_code(logits))
    if workspace is None:
        workspace = o.get("workspace")
    if workspace is None or workspace.numel() * workspace.element_size() < ws_bytes:
        workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    rc = _lib.load().aasd_verify_topk(
        logits.data_ptr(), _dtype_code(logits), B, C, k, V, row_stride, seq_stride,
        drafts.data_ptr(), draft_len.data_ptr(), int(topk),
        o["accept_len"].data_ptr(), o["best_cand"].data_ptr(), o["next_token"].data_ptr(),
        _ptr(o["row_argmax"]), _ptr(o["tok_pass"]), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _stream(dev))
    _check(rc)
    o["workspace"] = workspace
    return o


def build_tree(drafts: torch.Tensor, draft_len: torch.Tensor, strict: Optional[torch.Tensor] = None,
               draft_extras: Optional[torch.Tensor] = None, root_tok: Optional[torch.Tensor] = None,
               max_nodes: int = 64, want_mask: bool = True, want_cand_node: bool = True, out: Optional[dict] = None):
    """aasd_build_tree over drafts [B,C,k], draft_len [B,C], strict [B,C,k] u8, draft_extras [B,C,k,m].

    Returns a dict of device tensors: node_token, node_parent, node_depth [B,max_nodes] i32, node_strict u8,
    n_nodes [B], mask [B,max_nodes,W] (int32 storage of the u32 words), cand_node [B,C,k]."""
    _dev_check(drafts, draft_len, strict, draft_extras, root_tok)
    assert drafts.dtype == torch.int32 and drafts.is_contiguous() and drafts.dim() == 3
    assert draft_len.dtype == torch.int32 and draft_len.is_contiguous()
    B, C, k = drafts.shape
    m = 0
    if draft_extras is not None:
        assert draft_extras.dtype == torch.int32 and draft_extras.is_contiguous() and draft_extras.shape[:3] == (B, C, k)
        m = draft_extras.shape[3]
    if strict is not None:
        assert strict.dtype == torch.uint8 and strict.is_contiguous() and strict.shape == (B, C, k)
    if root_tok is not None:
        assert root_tok.dtype == torch.int32 and root_tok.is_contiguous() and root_tok.shape == (B,)
    dev = drafts.device
    o = dict(out or {})
    W = (max_nodes + 31) // 32
    def need(name, shape, dtype, wanted=True):
        if not wanted:
            o[name] = None
        elif o.get(name) is None:
            o[name] = torch.empty(shape, dtype=dtype, device=dev)
    need("node_token", (B, max_nodes), torch.int32)
    need("node_parent", (B, max_nodes), torch.int32)
    need("node_depth", (B, max_nodes), torch.int32)
    need("node_strict", (B, max_nodes), torch.uint8)
    need("n_nodes", (B,), torch.int32)
    need("mask", (B, max_nodes, W), torch.int32, want_mask)
    need("cand_node", (B, C, k), torch.int32, want_cand_node)
    rc = _lib.load().aasd_build_tree(
        drafts.data_ptr(), draft_len.data_ptr(), _ptr(strict), _ptr(draft_extras), m, _ptr(root_tok), B, C, k, max_nodes,
        o["node_token"].data_ptr(), o["node_parent"].data_ptr(), o["node_depth"].data_ptr(), o["node_strict"].data_ptr(),
        o["n_nodes"].data_ptr(), _ptr(o["mask"]), _ptr(o["cand_node"]), _stream(dev))
    _check(rc)
    return o


def verify_tree_workspace_bytes(B: int, N: int, V: int, dt: int) -> int:
    return int(_lib.load().aasd_verify_tree_workspace_bytes(B, N, V, dt))


def verify_tree(logits: torch.Tensor, node_token: torch.Tensor, node_parent: torch.Tensor, n_nodes: torch.Tensor,
                node_strict: Optional[torch.Tensor] = None, alpha: float = 0.1, beta: float = 0.1, flags: int = 0,
                V: Optional[int] = None, want_rows: bool = True, want_nodes: bool = True, want_near: bool = True,
                workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None):
    """aasd_verify_tree over logits[B, N, row_stride] and a tree of up to N nodes per sequence.

    Returns a dict of device tensors: accept_len, best_node, next_token [B]; accept_path [B,16]; row_entropy,
    row_pmax, row_argmax [B,N]; node_p, node_delta [B,N]; near_count [B] (the optional ones may be None)."""
    _dev_check(logits, node_token, node_parent, n_nodes, node_strict, workspace)
    assert logits.dim() == 3 and logits.stride(2) == 1
    B, N = logits.shape[0], logits.shape[1]
    for t in (node_token, node_parent):
        assert t.dtype == torch.int32 and t.is_contiguous() and t.shape == (B, N)
    assert n_nodes.dtype == torch.int32 and n_nodes.is_contiguous() and n_nodes.shape == (B,)
    if node_strict is not None:
        assert node_strict.dtype == torch.uint8 and node_strict.is_contiguous() and node_strict.shape == (B, N)
    row_stride = logits.stride(1)
    seq_stride = logits.stride(0) if B > 1 else N * row_stride
    V = logits.shape[2] if V is None else V
    dev = logits.device
    o = dict(out or {})
    def need(name, shape, dtype, wanted=True):
        if not wanted:
            o[name] = None
        elif o.get(name) is None:
            o[name] = torch.empty(shape, dtype=dtype, device=dev)
    need("accept_len", (B,), torch.int32)
    need("best_node", (B,), torch.int32)
    need("accept_path", (B, MAX_DRAFT), torch.int32)
    need("next_token", (B,), torch.int32)
    need("row_entropy", (B, N), torch.float32, want_rows)
    need("row_pmax", (B, N), torch.float32, want_rows)
    need("row_argmax", (B, N), torch.int32, want_rows)
    need("node_p", (B, N), torch.float32, want_nodes)
    need("node_delta", (B, N), torch.float32, want_nodes)
    need("near_count", (B,), torch.int32, want_near)
    ws_bytes = verify_tree_workspace_bytes(B, N, V, _dtype_code(logits))
    if workspace is None:
        workspace = o.get("workspace")
    if workspace is None or workspace.numel() * workspace.element_size() < ws_bytes:
        workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    rc = _lib.load().aasd_verify_tree(
        logits.data_ptr(), _dtype_code(logits), B, N, V, row_stride, seq_stride,
        node_token.data_ptr(), node_parent.data_ptr(), _ptr(node_strict), n_nodes.data_ptr(),
        float(alpha), float(beta), flags,
        o["accept_len"].data_ptr(), o["best_node"].data_ptr(), o["accept_path"].data_ptr(), o["next_token"].data_ptr(),
        _ptr(o["row_entropy"]), _ptr(o["row_pmax"]), _ptr(o["row_argmax"]), _ptr(o["node_p"]), _ptr(o["node_delta"]),
        _ptr(o["near_count"]), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(dev))
    _check(rc)
    o["workspace"] = workspace
    return o
