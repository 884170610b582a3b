"""ctypes binding of libslora.so -- argument marshalling only.

Every function has the name and argument order of its C declaration in include/slora.h
(the paper passages each call implements are cited there).  PyTorch is used for device
memory and the stream handle; no step of the method runs in Python or in torch ops.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslora.so")

SLORA_OK, SLORA_EINVAL, SLORA_ESTATE, SLORA_ENOSPC, SLORA_EHIP, SLORA_EZERO = 0, -1, -2, -3, -4, -5
PROJ = {"q": 0, "k": 1, "v": 2, "o": 3, "fc": 4, "pr": 5}
FROZEN = {"ln1_g": 0, "ln1_b": 1, "Wqkv": 2, "bqkv": 3, "Wo": 4, "bo": 5, "ln2_g": 6, "ln2_b": 7,
          "Wfc": 8, "bfc": 9, "Wpr": 10, "bpr": 11}
DTYPE_F32, DTYPE_BF16, DTYPE_MXFP8 = 0, 1, 2
MAX_RANK, MAX_CLIENTS = 16, 64

EXPORTS = ["slora_create", "slora_destroy", "slora_workspace_bytes", "slora_bind_workspace",
           "slora_bind_frozen", "slora_bind_adapter", "slora_server_fwd", "slora_server_bwd",
           "slora_adapter_step", "slora_fedavg", "slora_lora_linear_ws_bytes", "slora_lora_linear_fwd",
           "slora_lora_linear_bwd", "slora_strerror", "slora_last_hip_error", "slora_prof_enable",
           "slora_prof_read", "slora_frozen_linear_bf16", "slora_loss_head_ws_bytes",
           "slora_loss_head_prepare", "slora_loss_head", "slora_client_fwd", "slora_client_bwd",
           "slora_adapters_changed", "slora_adamw", "slora_mx_quantize", "slora_mx_dequantize",
           "slora_frozen_linear_mxfp8", "slora_mx_weight_bytes", "slora_mx_pack_weight",
           "slora_mx_lora_linear_ws_bytes", "slora_mx_lora_linear_fwd", "slora_mx_lora_linear_bwd",
           "slora_server_fwd_mx", "slora_server_bwd_mx", "slora_mx_quantize_fp4",
           "slora_frozen_linear_mxfp8_w4", "slora_lora_linear_bwd_noalloc", "slora_prof_read_kind", "slora_prof_read_clock"]
NOALLOC_SCRATCH_BYTES = 32 << 20
(PROF_GEMM, PROF_LN_FWD, PROF_LN_BWD, PROF_LORA_GRAD, PROF_SGD, PROF_ATTN_FWD, PROF_ATTN_BWD, PROF_FEDAVG,
 PROF_KINDS) = range(9)


class slora_config(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_head", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32), ("lora_r", ctypes.c_int32), ("lora_alpha", ctypes.c_float),
                ("lora_mask", ctypes.c_uint32), ("dtype", ctypes.c_int32), ("ln_eps", ctypes.c_float),
                ("max_seqs", ctypes.c_int32), ("seq_len", ctypes.c_int32)]


class SloraError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libslora error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """Load libslora.so (built by paper_2407_00952_amd.build); raises OSError if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libslora.so not built: run `python -m paper_2407_00952_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.slora_create.argtypes = [ctypes.POINTER(slora_config), ctypes.POINTER(vp)]
        L.slora_destroy.argtypes = [vp]
        L.slora_workspace_bytes.argtypes = [vp]
        L.slora_workspace_bytes.restype = sz
        L.slora_bind_workspace.argtypes = [vp, vp, sz]
        L.slora_bind_frozen.argtypes = [vp, i32, i32, vp]
        L.slora_bind_adapter.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.slora_server_fwd.argtypes = [vp, i32, vp, vp, vp, vp]
        L.slora_server_bwd.argtypes = [vp, vp, vp, vp]
        L.slora_adapter_step.argtypes = [vp, f32, vp]
        L.slora_fedavg.argtypes = [i32, vp, vp, sz, vp, vp]
        L.slora_lora_linear_ws_bytes.argtypes = [i32] * 5
        L.slora_lora_linear_ws_bytes.restype = sz
        L.slora_lora_linear_fwd.argtypes = [i32, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slora_lora_linear_bwd.argtypes = [i32, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slora_lora_linear_bwd_noalloc.argtypes = [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.slora_frozen_linear_bf16.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
        L.slora_client_fwd.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp]
        L.slora_client_bwd.argtypes = [vp, vp, vp]
        L.slora_adapters_changed.argtypes = [vp]
        L.slora_adamw.argtypes = [sz, vp, vp, vp, vp, f32, f32, f32, f32, f32, i32, vp]
        L.slora_loss_head_ws_bytes.argtypes = [i32, i32, i32]
        L.slora_loss_head_ws_bytes.restype = sz
        L.slora_loss_head_prepare.argtypes = [i32, i32, vp, vp, sz, vp]
        L.slora_loss_head.argtypes = [i32, i32, i32, vp, vp, vp, f32, vp, vp, sz, vp, vp, vp, vp]
        i64 = ctypes.c_int64
        L.slora_mx_quantize.argtypes = [i64, i32, vp, i64, vp, vp, vp]
        L.slora_mx_dequantize.argtypes = [i64, i32, vp, vp, vp, i64, vp]
        L.slora_frozen_linear_mxfp8.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.slora_mx_quantize_fp4.argtypes = [i64, i32, vp, i64, vp, vp, vp]
        L.slora_frozen_linear_mxfp8_w4.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.slora_server_fwd_mx.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.slora_server_bwd_mx.argtypes = [vp, vp, vp, vp, vp]
        L.slora_mx_weight_bytes.argtypes = [i32, i32]
        L.slora_mx_weight_bytes.restype = sz
        L.slora_mx_pack_weight.argtypes = [i32, i32, vp, vp, sz, vp]
        L.slora_mx_lora_linear_ws_bytes.argtypes = [i32, i32, i32, i32]
        L.slora_mx_lora_linear_ws_bytes.restype = sz
        L.slora_mx_lora_linear_fwd.argtypes = [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slora_mx_lora_linear_bwd.argtypes = [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slora_prof_enable.argtypes = [i32]
        L.slora_prof_read.argtypes = [vp, vp, vp]
        L.slora_prof_read_kind.argtypes = [i32, vp, vp, vp]
        L.slora_prof_read_clock.argtypes = [vp, vp]
        L.slora_strerror.argtypes = [i32]
        L.slora_strerror.restype = ctypes.c_char_p
        L.slora_last_hip_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        text = lib().slora_strerror(rc).decode()
        if rc == SLORA_EHIP:
            text += " (" + lib().slora_last_hip_error().decode() + ")"
        raise SloraError(rc, text)


def _p(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream


def _ptr_array(items):
    return (ctypes.c_void_p * len(items))(*[_p(t) for t in items])


# ---- same names as the C ABI -----------------------------------------------------------------
def slora_create(d_model, n_head, d_ff, n_blocks, lora_r, lora_alpha, lora_mask, max_seqs, seq_len,
                 dtype=DTYPE_BF16, ln_eps=1e-5):
    cfg = slora_config(d_model, n_head, d_ff, n_blocks, lora_r, lora_alpha, lora_mask, dtype, ln_eps,
                       max_seqs, seq_len)
    h = ctypes.c_void_p()
    _check(lib().slora_create(ctypes.byref(cfg), ctypes.byref(h)))
    return h


def slora_destroy(ctx):
    _check(lib().slora_destroy(ctx))


def slora_workspace_bytes(ctx):
    return int(lib().slora_workspace_bytes(ctx))


def slora_bind_workspace(ctx, ws, nbytes):
    _check(lib().slora_bind_workspace(ctx, _p(ws), nbytes))


def slora_bind_frozen(ctx, block, which, w):
    _check(lib().slora_bind_frozen(ctx, block, which, _p(w)))


def slora_bind_adapter(ctx, block, proj, A, B, dA, dB):
    _check(lib().slora_bind_adapter(ctx, block, proj, _p(A), _p(B), _p(dA), _p(dB)))


def slora_server_fwd(ctx, x_clients, batch, y, stream=None):
    K = len(x_clients)
    b = (ctypes.c_int32 * K)(*[int(v) for v in batch])
    _check(lib().slora_server_fwd(ctx, K, _ptr_array(x_clients), b, _p(y), _stream(stream)))


def slora_server_bwd(ctx, dy, dx_clients, stream=None):
    _check(lib().slora_server_bwd(ctx, _p(dy), _ptr_array(dx_clients), _stream(stream)))


def slora_server_fwd_mx(ctx, xq_clients, xs_clients, batch, y, stream=None):
    K = len(xq_clients)
    b = (ctypes.c_int32 * K)(*[int(v) for v in batch])
    _check(lib().slora_server_fwd_mx(ctx, K, _ptr_array(xq_clients), _ptr_array(xs_clients), b, _p(y),
                                     _stream(stream)))


def slora_server_bwd_mx(ctx, dy, dxq_clients, dxs_clients, stream=None):
    _check(lib().slora_server_bwd_mx(ctx, _p(dy), _ptr_array(dxq_clients), _ptr_array(dxs_clients), _stream(stream)))


def slora_adapter_step(ctx, lr, stream=None):
    _check(lib().slora_adapter_step(ctx, lr, _stream(stream)))


def slora_fedavg(client_params, sample_counts, n, out, stream=None):
    K = len(client_params)
    cnt = (ctypes.c_int64 * K)(*[int(v) for v in sample_counts])
    _check(lib().slora_fedavg(K, _ptr_array(client_params), cnt, n, _p(out), _stream(stream)))


def slora_lora_linear_ws_bytes(dtype, T, n_in, n_out, r):
    return int(lib().slora_lora_linear_ws_bytes(dtype, T, n_in, n_out, r))


def slora_lora_linear_fwd(dtype, T, n_in, n_out, r, alpha, x, W, bias, A, B, y, ws, ws_bytes, stream=None):
    _check(lib().slora_lora_linear_fwd(dtype, T, n_in, n_out, r, alpha, _p(x), _p(W), _p(bias), _p(A), _p(B),
                                       _p(y), _p(ws), ws_bytes, _stream(stream)))


def slora_lora_linear_bwd(dtype, T, n_in, n_out, r, alpha, x, dy, W, A, B, dx, dA, dB, ws, ws_bytes, stream=None):
    _check(lib().slora_lora_linear_bwd(dtype, T, n_in, n_out, r, alpha, _p(x), _p(dy), _p(W), _p(A), _p(B),
                                       _p(dx), _p(dA), _p(dB), _p(ws), ws_bytes, _stream(stream)))


def slora_lora_linear_bwd_noalloc(T, n_in, n_out, r, alpha, x, dy, W, A, B, dx, dA, dB, stream=None):
    _check(lib().slora_lora_linear_bwd_noalloc(T, n_in, n_out, r, alpha, _p(x), _p(dy), _p(W), _p(A), _p(B), _p(dx),
                                               _p(dA), _p(dB), _stream(stream)))


def slora_frozen_linear_bf16(T, n_in, n_out, x, W, bias, y, stream=None):
    _check(lib().slora_frozen_linear_bf16(T, n_in, n_out, _p(x), _p(W), _p(bias), _p(y), _stream(stream)))


def slora_mx_quantize(M, K, x, ldx, codes, scales, stream=None):
    _check(lib().slora_mx_quantize(M, K, _p(x), ldx, _p(codes), _p(scales), _stream(stream)))


def slora_mx_dequantize(M, K, codes, scales, y, ldy, stream=None):
    _check(lib().slora_mx_dequantize(M, K, _p(codes), _p(scales), _p(y), ldy, _stream(stream)))


def slora_frozen_linear_mxfp8(T, n_in, n_out, xq, xs, wq, ws, bias, y, stream=None):
    _check(lib().slora_frozen_linear_mxfp8(T, n_in, n_out, _p(xq), _p(xs), _p(wq), _p(ws), _p(bias), _p(y),
                                           _stream(stream)))


def slora_mx_quantize_fp4(M, K, x, ldx, codes, scales, stream=None):
    _check(lib().slora_mx_quantize_fp4(M, K, _p(x), ldx, _p(codes), _p(scales), _stream(stream)))


def slora_frozen_linear_mxfp8_w4(T, n_in, n_out, xq, xs, wq4, ws, bias, y, stream=None):
    _check(lib().slora_frozen_linear_mxfp8_w4(T, n_in, n_out, _p(xq), _p(xs), _p(wq4), _p(ws), _p(bias), _p(y),
                                              _stream(stream)))


def slora_mx_weight_bytes(n_in, n_out):
    return int(lib().slora_mx_weight_bytes(n_in, n_out))


def slora_mx_pack_weight(n_in, n_out, W, packed, nbytes, stream=None):
    _check(lib().slora_mx_pack_weight(n_in, n_out, _p(W), _p(packed), nbytes, _stream(stream)))


def slora_mx_lora_linear_ws_bytes(T, n_in, n_out, r):
    return int(lib().slora_mx_lora_linear_ws_bytes(T, n_in, n_out, r))


def slora_mx_lora_linear_fwd(T, n_in, n_out, r, alpha, x, packed_w, bias, A, B, y, ws, ws_bytes, stream=None):
    _check(lib().slora_mx_lora_linear_fwd(T, n_in, n_out, r, alpha, _p(x), _p(packed_w), _p(bias), _p(A), _p(B),
                                          _p(y), _p(ws), ws_bytes, _stream(stream)))


def slora_mx_lora_linear_bwd(T, n_in, n_out, r, alpha, x, dy, packed_w, A, B, dx, dA, dB, ws, ws_bytes, stream=None):
    _check(lib().slora_mx_lora_linear_bwd(T, n_in, n_out, r, alpha, _p(x), _p(dy), _p(packed_w), _p(A), _p(B),
                                          _p(dx), _p(dA), _p(dB), _p(ws), ws_bytes, _stream(stream)))


def slora_client_fwd(ctx, batch, tokens, vocab, wte, wpe, act, stream=None):
    _check(lib().slora_client_fwd(ctx, batch, _p(tokens), vocab, _p(wte), _p(wpe), _p(act), _stream(stream)))


def slora_client_bwd(ctx, dact, stream=None):
    _check(lib().slora_client_bwd(ctx, _p(dact), _stream(stream)))


def slora_adapters_changed(ctx):
    _check(lib().slora_adapters_changed(ctx))


def slora_adamw(n, p, g, m, v, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _check(lib().slora_adamw(n, _p(p), _p(g), _p(m), _p(v), lr, beta1, beta2, eps, weight_decay, step,
                             _stream(stream)))


def slora_loss_head_ws_bytes(max_tokens, d_model, vocab):
    return int(lib().slora_loss_head_ws_bytes(max_tokens, d_model, vocab))


def slora_loss_head_prepare(d_model, vocab, Wv, ws, ws_bytes, stream=None):
    _check(lib().slora_loss_head_prepare(d_model, vocab, _p(Wv), _p(ws), ws_bytes, _stream(stream)))


def slora_loss_head(T, d_model, vocab, y, lnf_g, lnf_b, eps, labels, ws, ws_bytes, loss_tok, loss, dy, stream=None):
    _check(lib().slora_loss_head(T, d_model, vocab, _p(y), _p(lnf_g), _p(lnf_b), eps, _p(labels), _p(ws), ws_bytes,
                                 _p(loss_tok), _p(loss), _p(dy), _stream(stream)))


def slora_prof_enable(kinds):
    _check(lib().slora_prof_enable(int(kinds)))


def slora_prof_read():
    """(gemm_ms, gemm_flop, launches) recorded since slora_prof_enable; blocks on the recorded events."""
    ms, fl, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    _check(lib().slora_prof_read(ctypes.byref(ms), ctypes.byref(fl), ctypes.byref(n)))
    return ms.value, fl.value, n.value


def slora_prof_read_clock():
    """(shader clock in MHz during the recorded GEMM launches, number of launches sampled); blocks."""
    mhz, n = ctypes.c_double(), ctypes.c_int()
    _check(lib().slora_prof_read_clock(ctypes.byref(mhz), ctypes.byref(n)))
    return mhz.value, n.value


def slora_prof_read_kind(kind):
    """(ms, work, launches) of one kind of kernel recorded since slora_prof_enable."""
    ms, wk, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    _check(lib().slora_prof_read_kind(int(kind), ctypes.byref(ms), ctypes.byref(wk), ctypes.byref(n)))
    return ms.value, wk.value, n.value


# ---- buffer management for tests and the benchmark (allocation + marshalling only) -----------------
def to_device_bf16(a):
    """float32 numpy array of bf16-representable values -> torch bf16 tensor on the GPU."""
    import torch
    from . import synth
    bits = synth.bf16_bits(a).reshape(np.shape(a))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_device_bf16(t):
    """torch bf16 tensor -> float32 numpy array."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


class Server:
    """Owns the device buffers of one server stack and forwards to the C ABI.

    blocks / adapters: as produced by synth.make_stack_inputs (numpy float32)."""

    def __init__(self, cfg, blocks, adapters, max_seqs=None, dtype=DTYPE_BF16):
        import torch
        self.cfg = cfg
        mask = 0
        for p in cfg.lora_proj:
            mask |= 1 << PROJ[p]
        self.max_seqs = max_seqs or cfg.n_seq
        self.ctx = slora_create(cfg.d_model, cfg.n_head, cfg.d_ff, len(blocks), cfg.lora_r, cfg.lora_alpha, mask,
                                self.max_seqs, cfg.seq_len, dtype, cfg.ln_eps)
        self.ws_bytes = slora_workspace_bytes(self.ctx)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device="cuda")
        base = self.ws.data_ptr()
        self._ws_ptr = (base + 255) & ~255
        slora_bind_workspace(self.ctx, self._ws_ptr, self.ws_bytes)
        self.frozen = []
        for l, blk in enumerate(blocks):
            dev = {k: to_device_bf16(v) for k, v in blk.items()}
            self.frozen.append(dev)
            for k, t in dev.items():
                slora_bind_frozen(self.ctx, l, FROZEN[k], t)
        # adapters live in ONE flat fp32 vector (block by block, projections in PROJ order, A then B): that
        # vector is what the aggregation of Eq. (8)-(9) averages; the gradients mirror the layout
        n_par = sum(int(np.size(A)) + int(np.size(Bm)) for ad in adapters for (A, Bm) in ad.values())
        self.flat = torch.empty(max(n_par, 1), dtype=torch.float32, device="cuda")
        self.flat_grad = torch.zeros(max(n_par, 1), dtype=torch.float32, device="cuda")
        self.adapters = []
        at = 0
        for l, ad in enumerate(adapters):
            dev = {}
            for p in sorted(ad.keys(), key=lambda k: PROJ[k]):
                A, Bm = ad[p]
                views = []
                for a in (A, Bm):
                    a = np.ascontiguousarray(a, dtype=np.float32)
                    v = self.flat[at:at + a.size].view(a.shape)
                    v.copy_(torch.from_numpy(a))
                    views.append((v, self.flat_grad[at:at + a.size].view(a.shape)))
                    at += a.size
                (tA, dA), (tB, dB) = views
                dev[p] = (tA, tB, dA, dB)
                slora_bind_adapter(self.ctx, l, PROJ[p], tA, tB, dA, dB)
            self.adapters.append(dev)
        self.n_params = n_par

    def fwd(self, x_clients, y, stream=None):
        slora_server_fwd(self.ctx, x_clients, [t.shape[0] for t in x_clients], y, stream)

    def bwd(self, dy, dx_clients, stream=None):
        slora_server_bwd(self.ctx, dy, dx_clients, stream)

    def fwd_mx(self, xq_clients, xs_clients, y, stream=None):
        slora_server_fwd_mx(self.ctx, xq_clients, xs_clients, [t.shape[0] for t in xq_clients], y, stream)

    def bwd_mx(self, dy, dxq_clients, dxs_clients, stream=None):
        slora_server_bwd_mx(self.ctx, dy, dxq_clients, dxs_clients, stream)

    def step(self, lr, stream=None):
        slora_adapter_step(self.ctx, lr, stream)

    def adapters_changed(self):
        slora_adapters_changed(self.ctx)

    def close(self):
        if self.ctx is not None:
            slora_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Client(Server):
    """One client's share of the model: embedding + its blocks with its own adapters (same C ABI context
    type as the server; the frozen tables wte / wpe are shared device tensors owned by the caller)."""

    def fwd(self, tokens, vocab, wte, wpe, act, stream=None):
        slora_client_fwd(self.ctx, act.shape[0], tokens, vocab, wte, wpe, act, stream)

    def bwd(self, dact, stream=None):
        slora_client_bwd(self.ctx, dact, stream)
