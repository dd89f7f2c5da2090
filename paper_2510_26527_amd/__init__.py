"""Python binding of libpsd (include/psd.h): argument marshalling only.

Every function has the name and the argument order of its C entry point and takes
torch tensors (device memory) where the C call takes device pointers; PyTorch is used for
allocation and streams, nothing is computed here.  There is no fallback: if the HIP
library has not been built (python -m paper_2510_26527_amd.build) or cannot be loaded,
the first call raises.
"""
import ctypes
import os

PSD_OK = 0
PSD_ERR_NULL, PSD_ERR_SHAPE, PSD_ERR_DTYPE, PSD_ERR_CAPACITY = -1, -2, -3, -4
PSD_ERR_TEMPERATURE, PSD_ERR_WORKSPACE, PSD_ERR_HIP, PSD_ERR_UNIMPLEMENTED = -5, -6, -7, -8
PSD_F32, PSD_BF16 = 0, 1
PSD_FLAG_NEAR_TIE, PSD_FLAG_ZERO_RESIDUAL = 1, 2
PSD_STATIC_SCRATCH_BYTES = 1 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpsd.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "psd.h")

_vp, _i32, _i64, _sz, _f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float


class psd_model_desc(ctypes.Structure):
    _fields_ = [("n_layers", _i32), ("d_model", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32),
                ("d_head", _i32), ("d_ffn", _i32), ("vocab", _i32), ("rope_theta", _f32),
                ("rms_eps", _f32), ("dtype", _i32)]


_SIGNATURES = {
    "psd_status_string": (ctypes.c_char_p, [_i32]),
    "psd_last_hip_error": (_i32, []),
    "psd_model_create": (_i32, [ctypes.POINTER(psd_model_desc), ctypes.POINTER(_vp), _i32, ctypes.POINTER(_vp)]),
    "psd_model_destroy": (_i32, [_vp]),
    "psd_model_create_w4": (_i32, [ctypes.POINTER(psd_model_desc), ctypes.POINTER(_vp), _i32, ctypes.POINTER(_vp),
                                   ctypes.POINTER(_vp), _i32, ctypes.POINTER(_vp)]),
    "psd_model_workspace_bytes": (_sz, [_vp, _i32, _i32, _i32]),
    "psd_model_packed_bytes": (_sz, [_vp]),
    "psd_model_pack": (_i32, [_vp, _vp, _sz, _vp]),
    "psd_kv_bytes": (_sz, [_vp, _i32, _i32]),
    "psd_kv_create": (_i32, [_vp, _i32, _i32, _vp, _vp, _vp, _i32, ctypes.POINTER(_vp)]),
    "psd_kv_destroy": (_i32, [_vp]),
    "psd_kv_len_upper_bound": (_i32, [_vp]),
    "psd_model_forward": (_i32, [_vp, _vp, _i32, _vp, _vp, _i32, _vp, _sz, _vp]),
    "psd_spec_accept_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "psd_spec_accept": (_i32, [_vp, _vp, _vp, _i32, _vp, _f32, _vp, _vp, _i32, _i32, _i32, _i32, _i64, _i64,
                               _vp, _vp, _sz, _vp]),
    "psd_spec_accept_static": (_i32, [_vp, _vp, _vp, _i32, _vp, _f32, _vp, _vp, _i32, _i32, _i32, _i32, _i64, _i64,
                                      _vp, _vp]),
    "psd_kv_truncate": (_i32, [_vp, _vp, _vp, _i32, _i32, _vp]),
    "psd_kv_truncate_to": (_i32, [_vp, _i32, _vp]),
    "psd_model_forward_tree": (_i32, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "psd_tree_accept": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _f32, _vp, _vp, _vp, _i32, _i32, _i32, _i64, _i64, _vp, _vp]),
    "psd_kv_compact_tree": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp]),
    "psd_probe_stream_read": (_i32, [_vp, _sz, _vp, _i32, _vp]),
    "psd_probe_mfma": (_i32, [_vp, _vp, _i32, _i32, _vp]),
    "psd_profile_enable": (_i32, [_i32]),
    "psd_profile_collect": (_i32, [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64)]),
}

PSD_KIND_NAMES = ("embed", "rmsnorm", "gemm_f32", "gemm_skinny", "gemm_tiled", "gemm_reduce", "rope_append", "attn",
                  "attn_combine", "swiglu", "lens", "accept_stats", "accept_draw", "accept_locate", "gemm_column", "gemm_w4",
                  "gemm_slot")

_lib = None


class PsdError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        extra = f", hipError {lib().psd_last_hip_error()}" if status == PSD_ERR_HIP else ""
        super().__init__(f"{where}: {status_string(status)} (status {status}{extra})")


def lib():
    """The loaded shared library; raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2510_26527_amd.build`; "
                               "there is no CPU fallback")
        import torch  # noqa: F401  loads the HIP runtime the library is linked against, before the library
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def status_string(status):
    return lib().psd_status_string(int(status)).decode()


def _check(status, where):
    if status != PSD_OK:
        raise PsdError(status, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream_ptr(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def dtype_code(torch_dtype):
    import torch
    return {torch.float32: PSD_F32, torch.bfloat16: PSD_BF16}[torch_dtype]


# ---------------------------------------------------------------- handles
def psd_model_create(desc: psd_model_desc, weight_ptrs):
    """weight_ptrs: device addresses (ints) in the header's order.  Returns the handle."""
    arr = (_vp * len(weight_ptrs))(*weight_ptrs)
    out = _vp()
    _check(lib().psd_model_create(ctypes.byref(desc), arr, len(weight_ptrs), ctypes.byref(out)), "psd_model_create")
    return out


def psd_model_create_w4(desc: psd_model_desc, weight_ptrs, scale_ptrs, zero_ptrs):
    """As psd_model_create; the projection pointers address 4-bit codes, scale_ptrs / zero_ptrs their group
    scales and zero points (7 per layer)."""
    arr = (_vp * len(weight_ptrs))(*weight_ptrs)
    sc = (_vp * len(scale_ptrs))(*scale_ptrs)
    zp = (_vp * len(zero_ptrs))(*zero_ptrs)
    out = _vp()
    _check(lib().psd_model_create_w4(ctypes.byref(desc), arr, len(weight_ptrs), sc, zp, len(scale_ptrs),
                                     ctypes.byref(out)), "psd_model_create_w4")
    return out


def psd_model_destroy(model):
    _check(lib().psd_model_destroy(model), "psd_model_destroy")


def psd_model_workspace_bytes(model, batch, n_new, max_len):
    return lib().psd_model_workspace_bytes(model, batch, n_new, max_len)


def psd_model_packed_bytes(model):
    return lib().psd_model_packed_bytes(model)


def psd_model_pack(model, packed_mem, stream=None):
    _check(lib().psd_model_pack(model, _ptr(packed_mem), packed_mem.numel() * packed_mem.element_size(),
                                _stream_ptr(stream)), "psd_model_pack")


def psd_kv_bytes(model, batch, max_len):
    return lib().psd_kv_bytes(model, batch, max_len)


def psd_kv_create(model, batch, max_len, k_mem, v_mem, lens_dev, len_upper_bound):
    out = _vp()
    _check(lib().psd_kv_create(model, batch, max_len, _ptr(k_mem), _ptr(v_mem), _ptr(lens_dev), len_upper_bound,
                               ctypes.byref(out)), "psd_kv_create")
    return out


def psd_kv_destroy(kv):
    _check(lib().psd_kv_destroy(kv), "psd_kv_destroy")


def psd_kv_len_upper_bound(kv):
    return lib().psd_kv_len_upper_bound(kv)


# ---------------------------------------------------------------- the hot path
def psd_model_forward(model, tokens_dev, n_new, kv, logits_out_dev, n_logit_rows, workspace, stream=None):
    _check(lib().psd_model_forward(model, _ptr(tokens_dev), n_new, kv, _ptr(logits_out_dev), n_logit_rows,
                                   _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream)), "psd_model_forward")


def psd_spec_accept_workspace_bytes(rows, gamma, n_p_rows, vocab):
    return lib().psd_spec_accept_workspace_bytes(rows, gamma, n_p_rows, vocab)


def psd_spec_accept(p_logits, q_logits, draft_tokens, gamma, uniforms, temperature, out_accept_len, out_token,
                    rows, n_p_rows, vocab, dtype, p_seq_stride, q_seq_stride, out_flags, workspace, stream=None):
    _check(lib().psd_spec_accept(_ptr(p_logits), _ptr(q_logits), _ptr(draft_tokens), gamma, _ptr(uniforms),
                                 float(temperature), _ptr(out_accept_len), _ptr(out_token), rows, n_p_rows, vocab,
                                 dtype, p_seq_stride, q_seq_stride, _ptr(out_flags), _ptr(workspace),
                                 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                 _stream_ptr(stream)), "psd_spec_accept")


def psd_spec_accept_static(p_logits, q_logits, draft_tokens, gamma, uniforms, temperature, out_accept_len, out_token,
                           rows, n_p_rows, vocab, dtype, p_seq_stride, q_seq_stride, out_flags, stream=None):
    _check(lib().psd_spec_accept_static(_ptr(p_logits), _ptr(q_logits), _ptr(draft_tokens), gamma, _ptr(uniforms),
                                        float(temperature), _ptr(out_accept_len), _ptr(out_token), rows, n_p_rows,
                                        vocab, dtype, p_seq_stride, q_seq_stride, _ptr(out_flags),
                                        _stream_ptr(stream)), "psd_spec_accept_static")


def psd_kv_truncate(kv, base_lens_dev, keep_dev, keep_offset, new_len_upper_bound=-1, stream=None):
    _check(lib().psd_kv_truncate(kv, _ptr(base_lens_dev), _ptr(keep_dev), keep_offset, new_len_upper_bound,
                                 _stream_ptr(stream)),
           "psd_kv_truncate")


def psd_kv_truncate_to(kv, new_len, stream=None):
    _check(lib().psd_kv_truncate_to(kv, new_len, _stream_ptr(stream)), "psd_kv_truncate_to")


def _host_i32(values):
    """A host int32 array for a `*_host` argument (the caller keeps it alive for the call)."""
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def psd_model_forward_tree(model, tokens_dev, n_nodes, parents, kv, logits_out_dev, workspace, stream=None):
    par = _host_i32(parents)
    _check(lib().psd_model_forward_tree(model, _ptr(tokens_dev), n_nodes, ctypes.cast(par, ctypes.c_void_p), kv,
                                        _ptr(logits_out_dev), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _stream_ptr(stream)), "psd_model_forward_tree")


def psd_tree_accept(p_logits, q_logits, tokens_dev, parents, n_nodes, uniforms, temperature, out_path_len, out_path,
                    out_token, rows, vocab, dtype, p_seq_stride, q_seq_stride, out_flags, stream=None):
    par = _host_i32(parents)
    _check(lib().psd_tree_accept(_ptr(p_logits), _ptr(q_logits), _ptr(tokens_dev), ctypes.cast(par, ctypes.c_void_p), n_nodes,
                                 _ptr(uniforms), float(temperature), _ptr(out_path_len), _ptr(out_path), _ptr(out_token),
                                 rows, vocab, dtype, p_seq_stride, q_seq_stride, _ptr(out_flags), _stream_ptr(stream)),
           "psd_tree_accept")


def psd_kv_compact_tree(kv, base_lens_dev, path_dev, path_len_dev, path_stride, n_nodes, new_len_upper_bound=-1,
                        stream=None):
    _check(lib().psd_kv_compact_tree(kv, _ptr(base_lens_dev), _ptr(path_dev), _ptr(path_len_dev), path_stride, n_nodes,
                                     new_len_upper_bound, _stream_ptr(stream)), "psd_kv_compact_tree")


def psd_probe_stream_read(src_dev, sink_dev, blocks, stream=None):
    _check(lib().psd_probe_stream_read(_ptr(src_dev), src_dev.numel() * src_dev.element_size(), _ptr(sink_dev), blocks,
                                       _stream_ptr(stream)), "psd_probe_stream_read")


def psd_probe_mfma(seed_dev, sink_dev, blocks, iters, stream=None):
    _check(lib().psd_probe_mfma(_ptr(seed_dev), _ptr(sink_dev), blocks, iters, _stream_ptr(stream)), "psd_probe_mfma")


def psd_profile_enable(max_launches):
    _check(lib().psd_profile_enable(max_launches), "psd_profile_enable")


def psd_profile_collect():
    """-> {kind name: (total milliseconds, launches)} for the launches recorded since the last call."""
    n = len(PSD_KIND_NAMES)
    ms = (ctypes.c_double * n)()
    cnt = (_i64 * n)()
    _check(lib().psd_profile_collect(ms, cnt), "psd_profile_collect")
    return {PSD_KIND_NAMES[k]: (ms[k], cnt[k]) for k in range(n)}
