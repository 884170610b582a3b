"""Host-side behaviour of the C ABI: the library loads, exports what include/slora.h declares,
and rejects bad arguments / call orders before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2407_00952_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000      # aligned, never dereferenced by the host-side checks


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "slora.h")).read()
    declared = set(re.findall(r"\b(slora_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_config_struct_layout_matches_header():
    # 11 four-byte fields in the declared order
    assert ctypes.sizeof(B.slora_config) == 44
    assert [f[0] for f in B.slora_config._fields_] == [
        "d_model", "n_head", "d_ff", "n_blocks", "lora_r", "lora_alpha", "lora_mask", "dtype", "ln_eps",
        "max_seqs", "seq_len"]


def _create(**kw):
    args = dict(d_model=128, n_head=2, d_ff=256, n_blocks=2, lora_r=4, lora_alpha=32.0, lora_mask=0b000101,
                max_seqs=4, seq_len=128)
    args.update(kw)
    return B.slora_create(**args)


@pytest.mark.parametrize("bad", [dict(d_model=100), dict(n_head=3), dict(d_ff=100), dict(n_blocks=0),
                                 dict(lora_r=0), dict(lora_r=17), dict(lora_mask=1 << 6), dict(max_seqs=0),
                                 dict(seq_len=100), dict(dtype=B.DTYPE_F32), dict(ln_eps=0.0),
                                 dict(d_model=4096, n_head=64), dict(dtype=3),
                                 # the compressed type needs widths that are multiples of 128
                                 dict(dtype=B.DTYPE_MXFP8, d_model=192, n_head=3),
                                 dict(dtype=B.DTYPE_MXFP8, d_ff=320)])
def test_create_rejects(bad):
    with pytest.raises(B.SloraError) as e:
        _create(**bad)
    assert e.value.code == B.SLORA_EINVAL


def test_compressed_context_needs_room_for_the_packed_weights():
    plain, comp = _create(), _create(dtype=B.DTYPE_MXFP8)
    d, dff, L, T = 128, 256, 2, 4 * 128
    packed = L * 2 * (3 * d * d + d * d + 2 * d * dff)           # 8 operands per block, one byte per weight
    extra = B.slora_workspace_bytes(comp) - B.slora_workspace_bytes(plain)
    assert packed <= extra <= packed * 1.2 + T * (max(dff, 3 * d) + d + dff) * 1.1 + 64 * 256
    B.slora_destroy(plain); B.slora_destroy(comp)


def test_workspace_and_binding_errors():
    ctx = _create()
    need = B.slora_workspace_bytes(ctx)
    assert need > 0 and need % 256 == 0
    assert B.slora_workspace_bytes(None) == 0
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_workspace(ctx, FAKE, need - 1)
    assert e.value.code == B.SLORA_ENOSPC
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_workspace(ctx, FAKE + 8, need)           # misaligned
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_frozen(ctx, 2, 0, FAKE)                  # block out of range
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_frozen(ctx, 0, 12, FAKE)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_adapter(ctx, 0, B.PROJ["k"], FAKE, FAKE, FAKE, FAKE)   # k is not in the mask
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_bind_adapter(ctx, 0, B.PROJ["q"], FAKE, None, FAKE, FAKE)
    assert e.value.code == B.SLORA_EINVAL
    B.slora_destroy(ctx)
    # a bigger model needs more
    big = _create(d_model=256, n_head=4, d_ff=1024)
    assert B.slora_workspace_bytes(big) > need
    B.slora_destroy(big)


def test_call_order_and_argument_checks():
    ctx = _create()
    y = FAKE
    # forward with nothing bound
    with pytest.raises(B.SloraError) as e:
        B.slora_server_fwd(ctx, [FAKE], [1], y, stream=0)
    assert e.value.code == B.SLORA_ESTATE
    # backward before forward, step before backward
    with pytest.raises(B.SloraError) as e:
        B.slora_server_bwd(ctx, FAKE, [FAKE], stream=0)
    assert e.value.code == B.SLORA_ESTATE
    with pytest.raises(B.SloraError) as e:
        B.slora_adapter_step(ctx, 0.1, stream=0)
    assert e.value.code == B.SLORA_ESTATE
    # argument errors are reported before state errors
    for clients, batch in (([], []), ([FAKE] * 65, [1] * 65), ([FAKE], [0]), ([FAKE, FAKE], [3, 2]), ([None], [1])):
        with pytest.raises(B.SloraError) as e:
            B.slora_server_fwd(ctx, clients, batch, y, stream=0)
        assert e.value.code == B.SLORA_EINVAL
    B.slora_destroy(ctx)


def test_fedavg_argument_checks():
    out = FAKE
    with pytest.raises(B.SloraError) as e:
        B.slora_fedavg([FAKE, FAKE], [0, 0], 16, out, stream=0)
    assert e.value.code == B.SLORA_EZERO
    with pytest.raises(B.SloraError) as e:
        B.slora_fedavg([FAKE, FAKE], [5, -1], 16, out, stream=0)
    assert e.value.code == B.SLORA_EZERO
    with pytest.raises(B.SloraError) as e:
        B.slora_fedavg([], [], 16, out, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_fedavg([FAKE] * 65, [1] * 65, 16, out, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    B.slora_fedavg([FAKE], [3], 0, out, stream=0)     # n = 0: nothing to do, no launch


def test_linear_argument_checks():
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_F32, 1024, 768, 768, 4) >= 2 * 4 * 1024 * 4
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, 1024, 768, 768, 4) > 0
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, 1024, 100, 768, 4) == 0      # in not a multiple of 64
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_F32, 1024, 768, 768, 17) == 0
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_fwd(B.DTYPE_F32, 16, 8, 8, 0, 32.0, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, 1 << 20,
                                stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_fwd(B.DTYPE_F32, 16, 8, 8, 2, 32.0, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, 16,
                                stream=0)
    assert e.value.code == B.SLORA_ENOSPC
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd(B.DTYPE_F32, 16, 8, 8, 2, 32.0, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                FAKE, 1 << 20, stream=0)
    assert e.value.code == B.SLORA_EINVAL


def test_documented_size_limits_are_enforced():
    # the frozen product: out a multiple of 8, in a multiple of 64, operands within 32-bit byte offsets
    for T, n_in, n_out in ((64, 64, 100), (64, 100, 64), (1 << 20, 4096, 64), (64, 65536, 65536)):
        with pytest.raises(B.SloraError) as e:
            B.slora_frozen_linear_bf16(T, n_in, n_out, FAKE, FAKE, None, FAKE, stream=0)
        assert e.value.code == B.SLORA_EINVAL, (T, n_in, n_out)
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, 64, 65536, 65536, 4) == 0
    # contexts: width above 2048, token count above 2^24, widest operand beyond 32-bit byte offsets
    for bad in (dict(d_model=2112, n_head=33), dict(max_seqs=1 << 16, seq_len=512),
                dict(d_model=2048, n_head=32, d_ff=8192, max_seqs=512, seq_len=1024)):
        with pytest.raises(B.SloraError) as e:
            _create(**bad)
        assert e.value.code == B.SLORA_EINVAL, bad
    B.slora_destroy(_create(d_model=2048, n_head=32, d_ff=8192, max_seqs=255, seq_len=1024))


def test_noalloc_backward_argument_checks():
    # checked before anything touches a GPU: sizes beyond the library's own scratch, bad pointers and sizes
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, 65536, 4096, 4096, 4) > B.NOALLOC_SCRATCH_BYTES
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd_noalloc(65536, 4096, 4096, 4, 32.0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                        stream=0)
    assert e.value.code == B.SLORA_ENOSPC
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd_noalloc(64, 100, 64, 4, 32.0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd_noalloc(64, 64, 64, 4, 32.0, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd_noalloc(64, 64, 64, 4, 32.0, FAKE + 8, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                        stream=0)
    assert e.value.code == B.SLORA_EINVAL


def test_measurement_hook_argument_checks():
    with pytest.raises(B.SloraError) as e:
        B.slora_prof_enable(1 << B.PROF_KINDS)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_prof_read_kind(B.PROF_KINDS)
    assert e.value.code == B.SLORA_EINVAL
    B.slora_prof_enable(0)
    assert B.slora_prof_read_kind(B.PROF_LN_FWD) == (0.0, 0.0, 0)


def test_loss_head_argument_checks():
    n = B.slora_loss_head_ws_bytes(32768, 1024, 50257)
    # two copies of the padded vocabulary matrix + one 16384-token chunk of bf16 logits + per-token buffers
    assert n >= 2 * 2 * 50304 * 1024 + 2 * 16384 * 50304 + 32768 * 1024 * (2 + 4 + 2)
    assert B.slora_loss_head_ws_bytes(32768, 1000, 50257) == 0       # d_model not a multiple of 64
    assert B.slora_loss_head_ws_bytes(32768, 1024, 70000) == 0       # vocabulary too large
    assert B.slora_loss_head_ws_bytes(0, 1024, 50257) == 0
    with pytest.raises(B.SloraError) as e:
        B.slora_loss_head_prepare(1024, 50257, None, FAKE, n, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_loss_head_prepare(1024, 50257, FAKE, FAKE, 1024, stream=0)
    assert e.value.code == B.SLORA_ENOSPC
    with pytest.raises(B.SloraError) as e:
        B.slora_loss_head(128, 1024, 50257, FAKE, FAKE, FAKE, 1e-5, None, FAKE, n, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.SLORA_EINVAL
    with pytest.raises(B.SloraError) as e:
        B.slora_loss_head(128, 1024, 50257, FAKE, FAKE, FAKE, 1e-5, FAKE, FAKE, 4096, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.SLORA_ENOSPC


def test_mx_argument_checks():
    """every check of the MXFP8 entry points precedes the first launch (include/slora.h)"""
    L = B.lib()
    ok = 4096          # a non-NULL, 16-byte aligned stand-in; no call below reaches a kernel
    assert L.slora_mx_quantize(4, 48, ok, 48, ok, ok, None) == B.SLORA_EINVAL            # K not a multiple of 32
    assert L.slora_mx_quantize(4, 64, ok, 32, ok, ok, None) == B.SLORA_EINVAL            # ldx < K
    assert L.slora_mx_quantize(4, 64, None, 64, ok, ok, None) == B.SLORA_EINVAL
    assert L.slora_mx_quantize(0, 64, ok, 64, ok, ok, None) == B.SLORA_EINVAL
    assert L.slora_mx_quantize(4, 64, ok + 2, 64, ok, ok, None) == B.SLORA_EINVAL        # misaligned source
    assert L.slora_mx_dequantize(4, 64, ok, ok, ok, 60, None) == B.SLORA_EINVAL
    assert L.slora_mx_dequantize(4, 64, ok, None, ok, 64, None) == B.SLORA_EINVAL
    assert L.slora_frozen_linear_mxfp8(8, 64, 8, ok, ok, ok, ok, None, ok, None) == B.SLORA_EINVAL    # n_in % 128
    assert L.slora_frozen_linear_mxfp8(8, 128, 12, ok, ok, ok, ok, None, ok, None) == B.SLORA_EINVAL  # n_out % 8
    assert L.slora_frozen_linear_mxfp8(8, 128, 8, ok, None, ok, ok, None, ok, None) == B.SLORA_EINVAL
    assert L.slora_frozen_linear_mxfp8(8, 128, 8, ok + 8, ok, ok, ok, None, ok, None) == B.SLORA_EINVAL
    assert L.slora_frozen_linear_mxfp8(1 << 22, 1024, 8, ok, ok, ok, ok, None, ok, None) == B.SLORA_EINVAL   # 2^32 bytes
    assert L.slora_mx_quantize_fp4(4, 48, ok, 48, ok, ok, None) == B.SLORA_EINVAL
    assert L.slora_mx_quantize_fp4(4, 64, ok, 64, ok + 2, ok, None) == B.SLORA_EINVAL
    assert L.slora_frozen_linear_mxfp8_w4(8, 64, 8, ok, ok, ok, ok, None, ok, None) == B.SLORA_EINVAL
    assert L.slora_frozen_linear_mxfp8_w4(8, 128, 8, ok, ok, None, ok, None, ok, None) == B.SLORA_EINVAL
    # compressed cut-layer traffic: the same checks as the bf16 calls plus the scale tables
    assert L.slora_server_fwd_mx(None, 1, ok, ok, ok, ok, None) == B.SLORA_EINVAL
    assert L.slora_server_bwd_mx(None, ok, ok, ok, None) == B.SLORA_EINVAL
    # the compressed LoRA layer
    assert L.slora_mx_weight_bytes(100, 128) == 0 and L.slora_mx_weight_bytes(128, 256) > 128 * 256 * 2
    assert L.slora_mx_lora_linear_ws_bytes(64, 128, 128, 17) == 0 and L.slora_mx_lora_linear_ws_bytes(64, 128, 128, 4) > 0
    assert L.slora_mx_pack_weight(128, 128, ok, ok, 16, None) == B.SLORA_ENOSPC
    assert L.slora_mx_pack_weight(128, 64, ok, ok, 1 << 20, None) == B.SLORA_EINVAL
    assert L.slora_mx_lora_linear_fwd(64, 128, 128, 4, 32.0, ok, ok, None, ok, ok, ok, ok, 16, None) == B.SLORA_ENOSPC
    assert L.slora_mx_lora_linear_fwd(64, 128, 128, 0, 32.0, ok, ok, None, ok, ok, ok, ok, 1 << 30, None) == B.SLORA_EINVAL
    assert L.slora_mx_lora_linear_bwd(64, 128, 128, 4, 32.0, ok, None, ok, ok, ok, ok, ok, ok, ok, 1 << 30, None) == B.SLORA_EINVAL


def test_strerror():
    L = B.lib()
    assert L.slora_strerror(0) == b"ok"
    assert b"workspace" in L.slora_strerror(B.SLORA_ENOSPC)
