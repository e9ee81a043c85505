"""Thin ctypes binding over librsd.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
data pointers and the current HIP stream to the C entry point of the same
name, and returns freshly allocated output tensors.  No arithmetic of the
method happens in Python.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librsd.so")

K_MAX = 16
NODES_MAX = 256
VOCAB_MAX = 65536
DTYPE_BF16, DTYPE_F32 = 0, 1
MODE_PATH, MODE_ALL_GROUPS = 0, 1
BASELINE_KSEQ, BASELINE_MULTIROUND = 0, 1
FLAG_DEGENERATE_RESIDUAL, FLAG_NONFINITE = 1, 2

_lib = None

_vp, _i32, _i64, _u32, _u64, _f32, _sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                           ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float,
                                           ctypes.c_size_t)

_SIGNATURES = {
    "rsd_version": (_i32, []),
    "rsd_status_string": (ctypes.c_char_p, [_i32]),
    "rsd_validate_tree": (_i32, [_vp, _i32]),
    "rsd_log_softmax_lse": (_i32, [_vp, _i64, _i32, _i32, _f32, _vp, _vp]),
    "rsd_gumbel_topk_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "rsd_gumbel_topk": (_i32, [_vp, _i64, _i32, _i32, _i32, _vp, _f32, _vp, _vp, _u64, _u32,
                               _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "rsd_sbs_step_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "rsd_sbs_step": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _f32, _u64, _u32,
                            _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "rsd_sbs_step_static": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _f32, _u64, _u32,
                                   _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "rsd_tree_attention_workspace_bytes": (_sz, [_i32] * 8),
    "rsd_tree_attention": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32,
                                  _i64, _i64, _i64, _vp, _vp, _vp, _f32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "rsd_tree_attention_layers_workspace_bytes": (_sz, [_i32] * 9),
    "rsd_tree_attention_layers": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i64, _i64, _i64, _i64,
                                         _i32, _i32, _i32, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp,
                                         _f32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "rsd_recursive_reject_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "rsd_recursive_reject": (_i32, [_vp, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _i32,
                                    _u64, _u32, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp,
                                    _vp, _sz, _vp]),
    "rsd_baseline_verify": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i32, _i32, _f32, _f32, _vp, _vp, _u64, _u32,
                                   _vp, _vp, _vp, _vp, _vp]),
    "rsd_filter_logits": (_i32, [_vp, _i64, _i32, _i32, _f32, _i32, _f32, _vp, _i64, _vp, _vp]),
    "rsd_filter_kv_cache": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i64, _i64, _i64,
                                   _vp, _vp, _i32, _vp, _vp, _vp, _vp]),
}


class RsdError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"rsd error {code}: {text}")
        self.code = code


def lib():
    """Load librsd.so once; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2402_14160_amd.build` "
                               "(or __graft_entry__.build()) first")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def _check(code):
    if code != 0:
        raise RsdError(code, lib().rsd_status_string(code).decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype=None):
    if not t.is_cuda:
        raise RuntimeError("rsd ops need tensors on the GPU; there is no CPU path")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t


def _opt_i32(t):
    return None if t is None else _dev(t, torch.int32)


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=device)


def validate_tree(parent_host):
    """Host check of one parent array (CPU int32 tensor or sequence)."""
    t = torch.as_tensor(parent_host, dtype=torch.int32).contiguous().cpu()
    return lib().rsd_validate_tree(ctypes.c_void_p(t.data_ptr()), t.numel())


def log_softmax_lse(logits, inv_temperature=1.0):
    if logits.dim() != 2 or logits.stride(1) != 1 or not logits.is_cuda or logits.dtype != torch.float32:
        raise ValueError("logits must be a 2-D fp32 GPU tensor with contiguous rows")
    R, V = logits.shape
    lse = torch.empty(R, dtype=torch.float32, device=logits.device)
    _check(lib().rsd_log_softmax_lse(_ptr(logits), logits.stride(0) if R > 1 else max(V, logits.stride(0)), R, V, inv_temperature,
                                     _ptr(lse), _stream()))
    return lse


def gumbel_topk(logits, k_max, k_per_row=None, inv_temperature=1.0, seq_id=None, node_id=None,
                seed=0, step=0, want_scores=True):
    """rsd_gumbel_topk; returns dict(tokens, perturbed, logprob, lse, count).  With
    want_scores=False only tokens and count are requested (the library then skips the
    row normaliser) and the three score entries are None."""
    if logits.dim() != 2 or logits.stride(1) != 1 or not logits.is_cuda or logits.dtype != torch.float32:
        raise ValueError("logits must be a 2-D fp32 GPU tensor with contiguous rows")
    R, V = logits.shape
    dev = logits.device
    tokens = torch.empty((R, k_max), dtype=torch.int32, device=dev)
    perturbed = torch.empty((R, k_max), dtype=torch.float32, device=dev) if want_scores else None
    logprob = torch.empty((R, k_max), dtype=torch.float32, device=dev) if want_scores else None
    lse = torch.empty(R, dtype=torch.float32, device=dev) if want_scores else None
    count = torch.empty(R, dtype=torch.int32, device=dev)
    _check(lib().rsd_gumbel_topk(_ptr(logits), logits.stride(0) if R > 1 else max(V, logits.stride(0)),
                                 R, V, k_max, _ptr(_opt_i32(k_per_row)), inv_temperature,
                                 _ptr(_opt_i32(seq_id)), _ptr(_opt_i32(node_id)), seed, step,
                                 _ptr(tokens), _ptr(perturbed), _ptr(logprob), _ptr(lse), _ptr(count),
                                 None, 0, _stream()))
    return dict(tokens=tokens, perturbed=perturbed, logprob=logprob, lse=lse, count=count)


def sbs_step(logits, sum_logprob, trunc_gumbel, n_in, width, inv_temperature=1.0, seq_id=None,
             node_id=None, seed=0, step=0, out=None, static_scratch=False):
    """rsd_sbs_step; returns dict(tokens, parent, sum_logprob, trunc_gumbel, n_out, lse).
    `out` (a dict as returned) makes the call write into existing tensors; with
    static_scratch=True the call goes to rsd_sbs_step_static, which takes no workspace, so that
    with `out` given nothing at all is allocated."""
    _dev(logits, torch.float32)
    _dev(sum_logprob, torch.float32)
    _dev(trunc_gumbel, torch.float32)
    _dev(n_in, torch.int32)
    B, W_in, V = logits.shape
    dev = logits.device
    if out is not None:
        tokens, parent, s_out, g_out = out["tokens"], out["parent"], out["sum_logprob"], out["trunc_gumbel"]
        n_out, lse = out["n_out"], out["lse"]
        for t, dt in ((tokens, torch.int32), (parent, torch.int32), (s_out, torch.float32),
                      (g_out, torch.float32), (n_out, torch.int32), (lse, torch.float32)):
            _dev(t, dt)
        if tokens.shape != (B, width) or lse.shape != (B, W_in):
            raise ValueError("output tensors do not fit this call")
    else:
        tokens = torch.empty((B, width), dtype=torch.int32, device=dev)
        parent = torch.empty((B, width), dtype=torch.int32, device=dev)
        s_out = torch.empty((B, width), dtype=torch.float32, device=dev)
        g_out = torch.empty((B, width), dtype=torch.float32, device=dev)
        n_out = torch.empty(B, dtype=torch.int32, device=dev)
        lse = torch.empty((B, W_in), dtype=torch.float32, device=dev)
    if static_scratch:
        _check(lib().rsd_sbs_step_static(_ptr(logits), _ptr(sum_logprob), _ptr(trunc_gumbel), _ptr(n_in),
                                         _ptr(_opt_i32(seq_id)), _ptr(_opt_i32(node_id)), B, W_in, V, width,
                                         inv_temperature, seed, step, _ptr(tokens), _ptr(parent), _ptr(s_out),
                                         _ptr(g_out), _ptr(n_out), _ptr(lse), _stream()))
        return dict(tokens=tokens, parent=parent, sum_logprob=s_out, trunc_gumbel=g_out,
                    n_out=n_out, lse=lse)
    nbytes = lib().rsd_sbs_step_workspace_bytes(B, W_in, V, width)
    ws = _workspace(nbytes, dev)
    _check(lib().rsd_sbs_step(_ptr(logits), _ptr(sum_logprob), _ptr(trunc_gumbel), _ptr(n_in),
                              _ptr(_opt_i32(seq_id)), _ptr(_opt_i32(node_id)), B, W_in, V, width,
                              inv_temperature, seed, step, _ptr(tokens), _ptr(parent), _ptr(s_out),
                              _ptr(g_out), _ptr(n_out), _ptr(lse), _ptr(ws), nbytes, _stream()))
    return dict(tokens=tokens, parent=parent, sum_logprob=s_out, trunc_gumbel=g_out,
                n_out=n_out, lse=lse)


def tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, prefix_len, n_nodes, parent, scale,
                   num_splits=0, return_lse=False, out=None, workspace=None):
    """rsd_tree_attention.  q [B,Hq,N,D]; k_prefix/v_prefix [B,Hkv,P,D] (any b/h/row strides,
    D contiguous) or None; k_tree/v_tree [B,Hkv,N,D]; returns out [B,Hq,N,D] fp32
    (rows >= n_nodes[b] are left untouched)."""
    dtype = {torch.bfloat16: DTYPE_BF16, torch.float32: DTYPE_F32}[q.dtype]
    _dev(q)
    _dev(k_tree, q.dtype)
    _dev(v_tree, q.dtype)
    _dev(prefix_len, torch.int32)
    _dev(n_nodes, torch.int32)
    _dev(parent, torch.int32)
    B, Hq, N, D = q.shape
    Hkv = k_tree.shape[1]
    if k_prefix is not None:
        if k_prefix.dtype != q.dtype or v_prefix.dtype != q.dtype or not k_prefix.is_cuda:
            raise TypeError("prefix K/V must match q's dtype and device")
        if k_prefix.stride(3) != 1 or v_prefix.stride() != k_prefix.stride():
            raise ValueError("prefix K and V need a contiguous last dim and identical strides")
        P_max = k_prefix.shape[2]
        sb, sh, sp = k_prefix.stride(0), k_prefix.stride(1), k_prefix.stride(2)
    else:
        P_max, sb, sh, sp = 0, 0, 0, D
    dev = q.device
    if out is None:
        out = torch.empty((B, Hq, N, D), dtype=torch.float32, device=dev)
    lse = torch.empty((B, Hq, N), dtype=torch.float32, device=dev) if return_lse else None
    nbytes = lib().rsd_tree_attention_workspace_bytes(dtype, B, Hq, Hkv, N, D, P_max, num_splits)
    ws = workspace if workspace is not None else _workspace(nbytes, dev)
    _check(lib().rsd_tree_attention(_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree),
                                    dtype, B, Hq, Hkv, N, D, P_max, sb, sh, sp, _ptr(prefix_len),
                                    _ptr(n_nodes), _ptr(parent), scale, num_splits, _ptr(out),
                                    _ptr(lse), _ptr(ws), ws.numel(), _stream()))
    return (out, lse) if return_lse else out


def tree_attention_layers(q, k_prefix, v_prefix, k_tree, v_tree, prefix_len, n_nodes, parent, scale,
                          num_splits=0, return_lse=False, out=None, workspace=None):
    """rsd_tree_attention_layers: q [L,B,Hq,N,D]; k_prefix/v_prefix [L,B,Hkv,P,D] (any layer/b/h/row
    strides, D contiguous) or None; k_tree/v_tree [L,B,Hkv,N,D]; prefix_len, n_nodes [B] and parent
    [B,N] are shared by the layers.  Returns out [L,B,Hq,N,D] fp32."""
    dtype = {torch.bfloat16: DTYPE_BF16, torch.float32: DTYPE_F32}[q.dtype]
    for t in (q, k_tree, v_tree):
        if not t.is_cuda or t.dtype != q.dtype or not t[0].is_contiguous():
            raise ValueError("q, k_tree, v_tree: GPU tensors of one dtype, contiguous inside a layer")
    if k_tree.stride(0) != v_tree.stride(0):
        raise ValueError("k_tree and v_tree need the same layer stride")
    _dev(prefix_len, torch.int32)
    _dev(n_nodes, torch.int32)
    _dev(parent, torch.int32)
    L, B, Hq, N, D = q.shape
    Hkv = k_tree.shape[2]
    if k_prefix is not None:
        if k_prefix.dtype != q.dtype or v_prefix.dtype != q.dtype or not k_prefix.is_cuda:
            raise TypeError("prefix K/V must match q's dtype and device")
        if k_prefix.stride(4) != 1 or v_prefix.stride() != k_prefix.stride():
            raise ValueError("prefix K and V need a contiguous last dim and identical strides")
        P_max = k_prefix.shape[3]
        sl, sb, sh, sp = k_prefix.stride(0), k_prefix.stride(1), k_prefix.stride(2), k_prefix.stride(3)
    else:
        P_max, sl, sb, sh, sp = 0, 0, 0, 0, D
    dev = q.device
    if out is None:
        out = torch.empty((L, B, Hq, N, D), dtype=torch.float32, device=dev)
    lse = torch.empty((L, B, Hq, N), dtype=torch.float32, device=dev) if return_lse else None
    nbytes = lib().rsd_tree_attention_layers_workspace_bytes(dtype, L, B, Hq, Hkv, N, D, P_max, num_splits)
    ws = workspace if workspace is not None else _workspace(nbytes, dev)
    _check(lib().rsd_tree_attention_layers(_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree),
                                           dtype, L, q.stride(0), sl, k_tree.stride(0), out.stride(0),
                                           lse.stride(0) if lse is not None else 0, B, Hq, Hkv, N, D, P_max,
                                           sb, sh, sp, _ptr(prefix_len), _ptr(n_nodes), _ptr(parent), scale,
                                           num_splits, _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream()))
    return (out, lse) if return_lse else out


def recursive_reject(draft_logits, target_logits, tokens, parent, n_nodes, inv_temperature=1.0,
                     mode=MODE_PATH, seq_id=None, seed=0, step=0, depth_max=None, diagnostics=True,
                     workspace=None):
    """rsd_recursive_reject; returns dict(accepted_nodes, accepted_tokens, n_accepted,
    last_token, final_node, theta, uniforms, flags)."""
    _dev(draft_logits, torch.float32)
    _dev(target_logits, torch.float32)
    _dev(tokens, torch.int32)
    _dev(parent, torch.int32)
    _dev(n_nodes, torch.int32)
    B, N, V = target_logits.shape
    dev = target_logits.device
    depth_max = N if depth_max is None else depth_max
    acc = torch.empty((B, depth_max), dtype=torch.int32, device=dev)
    acc_tok = torch.empty((B, depth_max), dtype=torch.int32, device=dev)
    n_acc = torch.empty(B, dtype=torch.int32, device=dev)
    last = torch.empty(B, dtype=torch.int32, device=dev)
    final_node = torch.empty(B, dtype=torch.int32, device=dev)
    theta = torch.empty((B, N), dtype=torch.float32, device=dev) if diagnostics else None
    uniforms = torch.empty((B, N), dtype=torch.float32, device=dev) if diagnostics else None
    flags = torch.empty(B, dtype=torch.int32, device=dev)
    nbytes = lib().rsd_recursive_reject_workspace_bytes(B, N, V)
    ws = workspace if workspace is not None else _workspace(nbytes, dev)
    _check(lib().rsd_recursive_reject(_ptr(draft_logits), _ptr(target_logits), B, N, V,
                                      inv_temperature, _ptr(tokens), _ptr(parent), _ptr(n_nodes),
                                      _ptr(_opt_i32(seq_id)), mode, seed, step, _ptr(acc),
                                      _ptr(acc_tok), depth_max, _ptr(n_acc), _ptr(last),
                                      _ptr(final_node), _ptr(theta), _ptr(uniforms), _ptr(flags),
                                      _ptr(ws), ws.numel(), _stream()))
    return dict(accepted_nodes=acc, accepted_tokens=acc_tok, n_accepted=n_acc, last_token=last,
                final_node=final_node, theta=theta, uniforms=uniforms, flags=flags)


def filter_kv_cache(k_cache, v_cache, k_tree, v_tree, prefix_len, accepted_nodes, n_accepted):
    """rsd_filter_kv_cache: appends the root's and the accepted nodes' rows of k_tree/v_tree
    [B,Hkv,N,D] to k_cache/v_cache [B,Hkv,capacity,D] (any b/h/row strides) in place;
    returns (new prefix_len [B], flags [B])."""
    dtype = {torch.bfloat16: DTYPE_BF16, torch.float32: DTYPE_F32}[k_cache.dtype]
    for t in (k_cache, v_cache):
        if not t.is_cuda or t.dtype != k_cache.dtype or t.stride(3) != 1:
            raise TypeError("cache tensors must be device tensors of one dtype with a contiguous last dim")
    if v_cache.stride() != k_cache.stride():
        raise ValueError("K and V cache need identical strides")
    _dev(k_tree, k_cache.dtype)
    _dev(v_tree, k_cache.dtype)
    _dev(prefix_len, torch.int32)
    _dev(accepted_nodes, torch.int32)
    _dev(n_accepted, torch.int32)
    B, H, cap, D = k_cache.shape
    N = k_tree.shape[2]
    L = accepted_nodes.shape[1]
    new_len = torch.empty(B, dtype=torch.int32, device=k_cache.device)
    flags = torch.empty(B, dtype=torch.int32, device=k_cache.device)
    _check(lib().rsd_filter_kv_cache(_ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree), dtype,
                                     B, H, N, D, cap, k_cache.stride(0), k_cache.stride(1),
                                     k_cache.stride(2), _ptr(prefix_len), _ptr(accepted_nodes), L,
                                     _ptr(n_accepted), _ptr(new_len), _ptr(flags), _stream()))
    return new_len, flags


def filter_logits(logits, inv_temperature=1.0, top_k=0, top_p=1.0, out=None, return_kept=False):
    """rsd_filter_logits on rows [R,V] (row-strided views allowed) or on contiguous [B,N,V]:
    entries outside the top-k / nucleus set become -inf.  `out=logits` filters in place."""
    def rows_of(t):
        if not t.is_cuda or t.dtype != torch.float32:
            raise TypeError("logits must be fp32 GPU tensors")
        if t.dim() == 3:
            if not t.is_contiguous():
                raise ValueError("a 3-D logits tensor must be contiguous")
            t = t.view(-1, t.shape[-1])
        if t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("logits rows must be contiguous")
        return t
    rows = rows_of(logits)
    R, V = rows.shape
    if out is None:
        ld = (V + 3) // 4 * 4
        out = torch.empty((R, ld), dtype=torch.float32, device=logits.device)[:, :V]
        out = out.view(logits.shape) if logits.dim() == 3 and ld == V else out
    orows = rows_of(out)
    if orows.shape != rows.shape:
        raise ValueError("out must have the shape of logits")
    stride = lambda t: t.stride(0) if R > 1 else max(V, t.stride(0))
    kept = torch.empty(R, dtype=torch.int32, device=logits.device) if return_kept else None
    _check(lib().rsd_filter_logits(_ptr(rows), stride(rows), R, V, inv_temperature, top_k, top_p,
                                   _ptr(orows), stride(orows), _ptr(kept), _stream()))
    return (out, kept) if return_kept else out


def baseline_verify(draft_logits, target_logits, drafts, method, gamma=1.0, inv_temperature=1.0,
                    seq_id=None, node_id=None, seed=0, step=0):
    """rsd_baseline_verify on rows [R,V] with drafts [R,K]; returns dict(accepted, token, theta, flags)."""
    for t in (draft_logits, target_logits):
        if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda or t.dtype != torch.float32:
            raise ValueError("logits must be 2-D fp32 GPU tensors with contiguous rows")
    if draft_logits.stride(0) != target_logits.stride(0) or draft_logits.shape != target_logits.shape:
        raise ValueError("draft and target rows need the same shape and row stride")
    _dev(drafts, torch.int32)
    R, V = target_logits.shape
    K = drafts.shape[1]
    dev = target_logits.device
    accepted = torch.empty(R, dtype=torch.int32, device=dev)
    token = torch.empty(R, dtype=torch.int32, device=dev)
    theta = torch.empty((R, K), dtype=torch.float32, device=dev)
    flags = torch.empty(R, dtype=torch.int32, device=dev)
    ld = target_logits.stride(0) if R > 1 else max(V, target_logits.stride(0))
    _check(lib().rsd_baseline_verify(_ptr(draft_logits), _ptr(target_logits), ld, R, V, _ptr(drafts), K, method,
                                     gamma, inv_temperature, _ptr(_opt_i32(seq_id)), _ptr(_opt_i32(node_id)),
                                     seed, step, _ptr(accepted), _ptr(token), _ptr(theta), _ptr(flags), _stream()))
    return dict(accepted=accepted, token=token, theta=theta, flags=flags)
