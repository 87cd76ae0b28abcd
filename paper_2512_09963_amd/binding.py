"""ctypes binding of the C-ABI library: argument marshalling only.

Every function here has the name and the semantics of the entry point it
wraps (see include/goodspeed.h).  torch is used for device memory and the
current stream; every step of the computation runs inside the library.
The library must have been built (python -m paper_2512_09963_amd.build);
loading fails loudly otherwise - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GS_LIB_PATH") or os.path.join(_HERE, "libgoodspeed.so")   # override: development builds

GS_F32, GS_BF16, GS_W4 = 0, 1, 2
_DTYPES = {"f32": GS_F32, "bf16": GS_BF16, "w4": GS_W4}
GS_ESHAPE = -2
_STATUS = {0: "GS_OK", -1: "GS_EINVAL", -2: "GS_ESHAPE", -3: "GS_ECAPACITY", -4: "GS_EDEVICE", -5: "GS_EUNSUPPORTED"}

EXPORTS = ["gs_last_error", "gs_accept_workspace_bytes", "gs_accept_reject", "gs_accept_reject_bf16", "gs_accept_reject_static",
           "gs_schedule_gamma", "gs_allocate_fixed", "gs_allocate_random",
           "gs_create", "gs_destroy", "gs_workspace_bytes", "gs_verify_batch", "gs_check_batch", "gs_profile_enable", "gs_profile_read", "gs_probe_stream_read", "gs_plan_attention", "gs_trace_residual", "gs_pack_weight", "gs_w4_packed_bytes", "gs_pack_weight_w4"]
STAGES = ["gemm", "attention", "glue", "accept"]


class GsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code


class gs_accept_out(C.Structure):
    _fields_ = [("accepted_len", C.c_void_p), ("next_token", C.c_void_p), ("accept_stat", C.c_void_p),
                ("ratio", C.c_void_p)]


class gs_model_desc(C.Structure):
    _fields_ = [(k, C.c_int) for k in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int)]


class gs_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)), ("wgu", C.POINTER(C.c_void_p)),
                ("wd", C.POINTER(C.c_void_p)), ("norm1", C.POINTER(C.c_void_p)), ("norm2", C.POINTER(C.c_void_p))]


class gs_kv_cache(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("page_size", C.c_int), ("n_pages", C.c_int)]


class gs_batch(C.Structure):
    _fields_ = [("n_servers", C.c_int), ("gamma_host", C.c_void_p), ("ctx_len_host", C.c_void_p),
                ("cu_rows", C.c_void_p), ("ctx_len", C.c_void_p), ("tokens", C.c_void_p),
                ("block_table", C.c_void_p), ("max_blocks", C.c_int), ("q_probs", C.c_void_p),
                ("u_accept", C.c_void_p), ("u_resample", C.c_void_p)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_09963_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.gs_last_error.restype = C.c_char_p
        L.gs_accept_workspace_bytes.restype = C.c_size_t
        L.gs_accept_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
        L.gs_accept_reject.restype = C.c_int
        L.gs_accept_reject.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.POINTER(gs_accept_out), C.c_void_p, C.c_size_t,
                                       C.c_void_p]
        L.gs_accept_reject_bf16.restype = C.c_int
        L.gs_accept_reject_bf16.argtypes = L.gs_accept_reject.argtypes
        L.gs_accept_reject_static.restype = C.c_int
        L.gs_accept_reject_static.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(gs_accept_out),
                                              C.c_void_p]
        L.gs_schedule_gamma.restype = C.c_int
        L.gs_schedule_gamma.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_double, C.c_double, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.gs_allocate_fixed.restype = C.c_int
        L.gs_allocate_fixed.argtypes = [C.c_int, C.c_int, C.c_void_p]
        L.gs_allocate_random.restype = C.c_int
        L.gs_allocate_random.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        if hasattr(L, "gs_create"):
            L.gs_create.restype = C.c_int
            L.gs_create.argtypes = [C.POINTER(gs_model_desc), C.POINTER(gs_weights), C.POINTER(C.c_void_p)]
            L.gs_destroy.restype = C.c_int
            L.gs_destroy.argtypes = [C.c_void_p]
            L.gs_workspace_bytes.restype = C.c_size_t
            L.gs_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
            L.gs_verify_batch.restype = C.c_int
            L.gs_verify_batch.argtypes = [C.c_void_p, C.POINTER(gs_kv_cache), C.POINTER(gs_batch),
                                          C.POINTER(gs_accept_out), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
            L.gs_check_batch.restype = C.c_int
            L.gs_check_batch.argtypes = [C.c_void_p, C.POINTER(gs_kv_cache), C.POINTER(gs_batch), C.c_void_p,
                                         C.c_size_t, C.c_void_p]
            L.gs_profile_enable.restype = C.c_int
            L.gs_profile_enable.argtypes = [C.c_void_p, C.c_int]
            L.gs_pack_weight.restype = C.c_int
            L.gs_pack_weight.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
            L.gs_w4_packed_bytes.restype = C.c_size_t
            L.gs_w4_packed_bytes.argtypes = [C.c_int, C.c_int]
            L.gs_pack_weight_w4.restype = C.c_int
            L.gs_pack_weight_w4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
            L.gs_trace_residual.restype = C.c_int
            L.gs_trace_residual.argtypes = [C.c_void_p, C.c_void_p]
            L.gs_probe_stream_read.restype = C.c_int
            L.gs_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
            L.gs_plan_attention.restype = C.c_int
            L.gs_plan_attention.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
            L.gs_profile_read.restype = C.c_int
            L.gs_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(code):
    if code != 0:
        raise GsError(code, lib().gs_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _host_i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def gs_accept_workspace_bytes(n_servers, n_rows, vocab):
    return int(lib().gs_accept_workspace_bytes(n_servers, n_rows, vocab))


def make_accept_out(n_servers, n_draft, device, want_ratio=True):
    """Device output buffers of gs_accept_reject / gs_verify_batch as a dict of tensors."""
    out = {"accepted_len": torch.empty(n_servers, dtype=torch.int32, device=device),
           "next_token": torch.empty(n_servers, dtype=torch.int32, device=device),
           "accept_stat": torch.empty(n_servers, dtype=torch.float32, device=device),
           "ratio": torch.empty(max(n_draft, 1), dtype=torch.float32, device=device)[:n_draft] if want_ratio else None}
    return out


def _accept_out_struct(out):
    return gs_accept_out(_ptr(out["accepted_len"]), _ptr(out["next_token"]), _ptr(out["accept_stat"]),
                         _ptr(out.get("ratio")))


def gs_accept_reject(gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens, u_accept, u_resample,
                     out, workspace, stream=None):
    """Enqueues accept/reject + resample; `out` is a dict from make_accept_out, `workspace` a uint8 device tensor."""
    g = _host_i32(gamma_host)
    st = _accept_out_struct(out)
    _check(lib().gs_accept_reject(int(g.size), g.ctypes.data, _ptr(cu_rows), int(vocab), _ptr(target_logits),
                                  _ptr(q_probs), _ptr(draft_tokens), _ptr(u_accept), _ptr(u_resample),
                                  C.byref(st), _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                  _stream(stream)))
    return out


def gs_accept_reject_bf16(gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens, u_accept, u_resample,
                          out, workspace, stream=None):
    """gs_accept_reject on bfloat16 target_logits and q_probs (device tensors of dtype bfloat16)."""
    assert target_logits.dtype == torch.bfloat16 and (q_probs is None or q_probs.dtype == torch.bfloat16)
    g = _host_i32(gamma_host)
    st = _accept_out_struct(out)
    _check(lib().gs_accept_reject_bf16(int(g.size), g.ctypes.data, _ptr(cu_rows), int(vocab), _ptr(target_logits),
                                       _ptr(q_probs), _ptr(draft_tokens), _ptr(u_accept), _ptr(u_resample),
                                       C.byref(st), _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                       _stream(stream)))
    return out


def gs_accept_reject_static(gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens, u_accept, u_resample,
                            out, stream=None):
    """gs_accept_reject on the library's static scratch array: no workspace argument, nothing allocated."""
    g = _host_i32(gamma_host)
    st = _accept_out_struct(out)
    _check(lib().gs_accept_reject_static(int(g.size), g.ctypes.data, _ptr(cu_rows), int(vocab), _ptr(target_logits),
                                         _ptr(q_probs), _ptr(draft_tokens), _ptr(u_accept), _ptr(u_resample),
                                         C.byref(st), _stream(stream)))
    return out


def gs_schedule_gamma(accepted_len, accept_stat, gamma_prev, alpha_hat, x_smooth, eta, beta, capacity,
                      gamma_min=0, gamma_max=-1):
    """Updates alpha_hat and x_smooth (float64 numpy arrays) IN PLACE and returns gamma_next (int32 array)."""
    m = _host_i32(accepted_len)
    st = np.ascontiguousarray(accept_stat, dtype=np.float32)
    gp = _host_i32(gamma_prev)
    n = int(gp.size)
    assert alpha_hat.dtype == np.float64 and x_smooth.dtype == np.float64
    assert alpha_hat.flags.c_contiguous and x_smooth.flags.c_contiguous
    nxt = np.zeros(n, dtype=np.int32)
    _check(lib().gs_schedule_gamma(n, m.ctypes.data, st.ctypes.data, gp.ctypes.data, alpha_hat.ctypes.data,
                                   x_smooth.ctypes.data, float(eta), float(beta), int(capacity), int(gamma_min),
                                   int(gamma_max), nxt.ctypes.data))
    return nxt


def gs_allocate_fixed(n, capacity):
    """Fixed-S: the even split of the capacity (int32 array [n])."""
    nxt = np.zeros(int(n), dtype=np.int32)
    _check(lib().gs_allocate_fixed(int(n), int(capacity), nxt.ctypes.data))
    return nxt


def gs_allocate_random(n, capacity, uniforms):
    """Random-S: slot k goes to server floor(uniforms[k] * n) (int32 array [n])."""
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    if u.size < int(capacity):
        raise ValueError("one uniform per draft slot is needed")
    nxt = np.zeros(int(n), dtype=np.int32)
    _check(lib().gs_allocate_random(int(n), int(capacity), u.ctypes.data, nxt.ctypes.data))
    return nxt


def gs_plan_attention(n_kv_heads, group, gamma, ctx_len):
    """Host-only: (steps_per_split, n_workgroups, busiest_cu_steps) of the attention launch for this geometry."""
    g = np.ascontiguousarray(gamma, dtype=np.int32)
    c = np.ascontiguousarray(ctx_len, dtype=np.int32)
    if g.shape != c.shape:
        raise ValueError("gamma and ctx_len must have one entry per server")
    sps, n, busy = C.c_int(0), C.c_long(0), C.c_long(0)
    _check(lib().gs_plan_attention(int(n_kv_heads), int(group), int(g.size), g.ctypes.data, c.ctypes.data,
                                   C.addressof(sps), C.addressof(n), C.addressof(busy)))
    return sps.value, n.value, busy.value


def gs_probe_stream_read(src, sink, stream=None):
    """Enqueues the plain streaming-read probe over the device tensor `src` (sink: >= 64 KiB device tensor)."""
    _check(lib().gs_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))


def gs_pack_weight_w4(codes, scales, zeros, stream=None):
    """codes uint8 [N, K], scales bf16 [N, K/128], zeros uint8 [N, K/128] (device tensors) -> packed uint8
    device tensor in the layout the 4-bit projection kernel streams."""
    n, k = int(codes.shape[0]), int(codes.shape[1])
    nbytes = int(lib().gs_w4_packed_bytes(n, k))
    if nbytes == 0:
        raise GsError(GS_ESHAPE, "4-bit matrices need n_out to be a multiple of 64 and k_in of 128")
    out = torch.empty(nbytes, dtype=torch.uint8, device=codes.device)
    _check(lib().gs_pack_weight_w4(_ptr(codes), _ptr(scales), _ptr(zeros), _ptr(out), n, k, _stream(stream)))
    return out


def gs_pack_weight(w, stream=None):
    """Returns a new device tensor holding the [out, in] matrix `w` in the library's projection layout."""
    out = torch.empty_like(w)
    dtype = GS_BF16 if w.dtype == torch.bfloat16 else GS_F32
    _check(lib().gs_pack_weight(_ptr(w), _ptr(out), int(w.shape[0]), int(w.shape[1]), dtype, _stream(stream)))
    return out


class Verifier:
    """Owns a gs_ctx: model description plus device weight pointers (tensors are kept alive here)."""

    def __init__(self, desc: dict, top: dict, layers: list):
        """desc: fields of gs_model_desc (dtype as 'f32' | 'bf16' | 'w4'); top: embed, lm_head, final_norm tensors;
        layers: list of dicts wqkv, wo, wgu, wd, norm1, norm2 (device tensors)."""
        self.desc = dict(desc)
        self._keep = (top, layers)
        d = gs_model_desc(desc["n_layers"], desc["d_model"], desc["n_heads"], desc["n_kv_heads"], desc["head_dim"],
                          desc["d_ffn"], desc["vocab"], desc["rope_theta"], desc["rms_eps"],
                          _DTYPES[desc["dtype"]])
        n = desc["n_layers"]
        arr = {k: (C.c_void_p * n)(*[layers[l][k].data_ptr() for l in range(n)])
               for k in ("wqkv", "wo", "wgu", "wd", "norm1", "norm2")}
        w = gs_weights(_ptr(top["embed"]), _ptr(top["lm_head"]), _ptr(top["final_norm"]),
                       *[C.cast(arr[k], C.POINTER(C.c_void_p)) for k in ("wqkv", "wo", "wgu", "wd", "norm1", "norm2")])
        self._ctx = C.c_void_p()
        _check(lib().gs_create(C.byref(d), C.byref(w), C.byref(self._ctx)))

    def close(self):
        if self._ctx:
            lib().gs_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def gs_trace_residual(self, trace):
        """trace: float32 device tensor [(n_layers + 1), R, d_model] or None."""
        self._trace = trace
        _check(lib().gs_trace_residual(self._ctx, _ptr(trace)))

    def gs_profile_enable(self, on):
        _check(lib().gs_profile_enable(self._ctx, 1 if on else 0))

    def gs_profile_read(self):
        """dict stage -> (milliseconds, launches) since the last read."""
        ms = (C.c_double * len(STAGES))()
        cnt = (C.c_long * len(STAGES))()
        _check(lib().gs_profile_read(self._ctx, ms, cnt))
        return {s: (ms[i], cnt[i]) for i, s in enumerate(STAGES)}

    def gs_workspace_bytes(self, max_rows, max_servers, max_ctx):
        return int(lib().gs_workspace_bytes(self._ctx, max_rows, max_servers, max_ctx))

    def gs_check_batch(self, k_pages, v_pages, page_size, n_pages, gamma_host, ctx_len_host, cu_rows, ctx_len, tokens,
                       block_table, workspace, stream=None):
        """Debug check of the device-resident descriptor; raises GsError(GS_EINVAL) naming the first violation."""
        g = _host_i32(gamma_host)
        cl = _host_i32(ctx_len_host)
        kv = gs_kv_cache(_ptr(k_pages), _ptr(v_pages), int(page_size), int(n_pages))
        b = gs_batch(int(g.size), g.ctypes.data, cl.ctypes.data, _ptr(cu_rows).value, _ptr(ctx_len).value,
                     _ptr(tokens).value, _ptr(block_table).value, int(block_table.shape[1]), None, None, None)
        _check(lib().gs_check_batch(self._ctx, C.byref(kv), C.byref(b), _ptr(workspace), workspace.numel(),
                                    _stream(stream)))

    def gs_verify_batch(self, k_pages, v_pages, page_size, n_pages, gamma_host, ctx_len_host, cu_rows, ctx_len,
                        tokens, block_table, q_probs, u_accept, u_resample, out, logits_out, workspace, stream=None):
        g = _host_i32(gamma_host)
        cl = _host_i32(ctx_len_host)
        kv = gs_kv_cache(_ptr(k_pages), _ptr(v_pages), int(page_size), int(n_pages))
        b = gs_batch(int(g.size), g.ctypes.data, cl.ctypes.data, _ptr(cu_rows).value, _ptr(ctx_len).value,
                     _ptr(tokens).value, _ptr(block_table).value, int(block_table.shape[1]),
                     None if q_probs is None else q_probs.data_ptr(),
                     None if u_accept is None else u_accept.data_ptr(),
                     None if u_resample is None else u_resample.data_ptr())
        st = _accept_out_struct(out) if out is not None else None
        _check(lib().gs_verify_batch(self._ctx, C.byref(kv), C.byref(b), C.byref(st) if st is not None else None,
                                     _ptr(logits_out), _ptr(workspace), workspace.numel(), _stream(stream)))
        return out
