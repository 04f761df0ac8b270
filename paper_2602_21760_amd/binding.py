"""Thin ctypes binding of libhyb.so: argument marshalling only.  Every function has the name of
the C entry point it calls (see include/hyb.h); tensors are torch CUDA tensors used purely as
device memory, work is enqueued on torch's current stream.  Loading fails loudly if the
library has not been built: there is no fallback path."""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhyb.so")

HYB_F32, HYB_BF16 = 0, 1
HYB_NORM_L1, HYB_NORM_L2 = 1, 2
HYB_EPI_BIAS, HYB_EPI_GELU_TANH, HYB_EPI_SILU, HYB_EPI_GATE_RESIDUAL, HYB_EPI_GEGLU = 0, 1, 2, 3, 5
STATUS = {0: "HYB_OK", 1: "HYB_ERR_NULL", 2: "HYB_ERR_SHAPE", 3: "HYB_ERR_DTYPE", 4: "HYB_ERR_ALIGN",
          5: "HYB_ERR_WORKSPACE", 6: "HYB_ERR_LAUNCH"}


class HybError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s: %s" % (STATUS.get(code, code), msg))
        self.code = code


class BlockDesc(C.Structure):
    _fields_ = [("batch", C.c_int), ("n_img", C.c_int), ("n_txt", C.c_int), ("hidden", C.c_int),
                ("heads", C.c_int), ("head_dim", C.c_int), ("mlp_ratio", C.c_int), ("dtype", C.c_int),
                ("ln_eps", C.c_float), ("txt_pre_only", C.c_int)]


class StreamWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_out", "w_fc1", "w_fc2", "b_qkv", "b_out", "b_fc1", "b_fc2")]


class BlockWeights(C.Structure):
    _fields_ = [("img", StreamWeights), ("txt", StreamWeights)]


class SdxlBlockDesc(C.Structure):
    _fields_ = [("batch", C.c_int), ("tokens", C.c_int), ("channels", C.c_int), ("heads", C.c_int),
                ("head_dim", C.c_int), ("n_ctx", C.c_int), ("ctx_dim", C.c_int), ("groups", C.c_int),
                ("dtype", C.c_int), ("gn_eps", C.c_float), ("ln_eps", C.c_float)]


SDXL_WEIGHT_FIELDS = ("gn_g", "gn_b", "ln1_g", "ln1_b", "ln2_g", "ln2_b", "ln3_g", "ln3_b", "w_qkv1", "w_o1", "b_o1",
                      "w_q2", "w_kv2", "w_o2", "b_o2", "w_ff1", "b_ff1", "w_ff2", "b_ff2")


class SdxlBlockWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in SDXL_WEIGHT_FIELDS]


HYB_SWITCH_MAX_STEPS = 1024


class SwitchState(C.Structure):
    _fields_ = [("total_steps", C.c_int), ("window", C.c_int), ("tau_cap", C.c_int), ("k", C.c_int),
                ("g_slope", C.c_float), ("step", C.c_int), ("tau1", C.c_int), ("tau2", C.c_int),
                ("history", C.c_double * HYB_SWITCH_MAX_STEPS)]


_vp, _i, _f, _sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
SIGNATURES = {
    "hyb_version": (C.c_int, []),
    "hyb_last_error_string": (C.c_char_p, []),
    "hyb_cfg_combine": (_i, [_vp, _vp, _vp, _sz, _f, _i, _vp]),
    "hyb_branch_discrepancy": (_i, [_vp, _vp, _i, _sz, _i, _i, _vp, _vp, _sz, _vp]),
    "hyb_discrepancy_workspace_bytes": (_sz, [_i, _sz]),
    "hyb_euler_step": (_i, [_vp, _vp, _vp, _sz, _f, _f, _i, _i, _vp]),
    "hyb_cfg_disc_euler": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _sz, _f, _f, _f, _vp, _vp, _i, _vp, _sz, _vp]),
    "hyb_cfg_disc_affine": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _sz, _f, _f, _f, _vp, _vp, _i, _vp, _sz, _vp]),
    "hyb_cfg_disc_euler_noalloc": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _sz, _f, _f, _f, _vp, _vp, _i, _vp]),
    "hyb_joint_attention": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _vp]),
    "hyb_joint_attention_ws": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _vp, _sz, _vp]),
    "hyb_joint_attention_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "hyb_joint_attention_prescaled": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]),
    "hyb_adaln_modulation": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "hyb_layernorm_modulate": (_i, [_vp, _vp, _vp, _sz, _vp, _i, _i, _i, _f, _i, _vp]),
    "hyb_linear": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _i, _sz, _vp]),
    "hyb_block_forward": (_i, [C.POINTER(BlockDesc), C.POINTER(BlockWeights), _vp, _vp, _vp, _vp, _sz, _vp, _vp,
                               _vp, _sz, _vp]),
    "hyb_block_workspace_bytes": (_sz, [C.POINTER(BlockDesc)]),
    "hyb_timestep_embedding": (_i, [_vp, _vp, _i, _i, _i, _vp]),
    "hyb_patchify": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "hyb_unpatchify": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp]),
    "hyb_convert": (_i, [_vp, _vp, _sz, _i, _vp]),
    "hyb_groupnorm": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _vp, _sz, _vp]),
    "hyb_groupnorm_workspace_bytes": (_sz, [_i, _i]),
    "hyb_layernorm_affine": (_i, [_vp, _vp, _vp, _vp, _i, _i, _f, _i, _vp]),
    "hyb_sdxl_block_forward": (_i, [C.POINTER(SdxlBlockDesc), C.POINTER(SdxlBlockWeights), _vp, _vp, _vp, _vp, _sz, _vp]),
    "hyb_sdxl_block_workspace_bytes": (_sz, [C.POINTER(SdxlBlockDesc)]),
    "hyb_switch_init": (_i, [C.POINTER(SwitchState), _i, _i, _f, _i, _i]),
    "hyb_switch_push": (_i, [C.POINTER(SwitchState), _f, C.POINTER(C.c_int)]),
    "hyb_switch_stage": (_i, [C.POINTER(SwitchState), _i]),
    "hyb_trace_enable": (_i, [_i]),
    "hyb_trace_summary": (_i, [C.c_char_p, _sz]),
}

_lib = None


def lib():
    """The loaded library (loads on first use; raises if libhyb.so is missing)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libhyb.so is not built (%s missing): run `python -m paper_2602_21760_amd.build` "
                               "or __graft_entry__.build(); there is no fallback path" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise HybError(rc, lib().hyb_last_error_string().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t):
    if t.dtype == torch.float32:
        return HYB_F32
    if t.dtype == torch.bfloat16:
        return HYB_BF16
    raise TypeError("unsupported tensor dtype %s" % t.dtype)


def _p(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def hyb_version():
    return lib().hyb_version()


def hyb_cfg_combine(v_c, v_u, v_out, scale):
    _check(lib().hyb_cfg_combine(_p(v_c), _p(v_u, v_c.dtype), _p(v_out, v_c.dtype), v_c.numel(), scale, _dt(v_c),
                                 _stream()))
    return v_out


def hyb_discrepancy_workspace_bytes(batch, n_per_sample):
    return lib().hyb_discrepancy_workspace_bytes(batch, n_per_sample)


def hyb_branch_discrepancy(v_c, v_u, p, out, workspace):
    """v_c, v_u: [batch, ...]; out: float32[batch]."""
    batch = v_c.shape[0]
    n = v_c.numel() // batch if batch else 0
    _check(lib().hyb_branch_discrepancy(_p(v_c), _p(v_u, v_c.dtype), batch, n, p, _dt(v_c), _p(out, torch.float32),
                                        _p(workspace), _nbytes(workspace), _stream()))
    return out


def hyb_euler_step(x, v, x_out, t, t_next):
    _check(lib().hyb_euler_step(_p(x), _p(v), _p(x_out, x.dtype), x.numel(), t, t_next, _dt(x), _dt(v), _stream()))
    return x_out


def hyb_cfg_disc_euler(v_c, v_u, x, x_out, scale, t, t_next, disc_l1=None, disc_l2=None, workspace=None,
                       x_out_lowp=None, v_out=None):
    batch = v_c.shape[0]
    n = v_c.numel() // batch if batch else 0
    _check(lib().hyb_cfg_disc_euler(_p(v_c), _p(v_u, v_c.dtype), _p(x, torch.float32), _p(x_out, torch.float32),
                                    _p(x_out_lowp, torch.bfloat16), _p(v_out, v_c.dtype), batch, n, scale, t, t_next,
                                    _p(disc_l1, torch.float32), _p(disc_l2, torch.float32), _dt(v_c),
                                    _p(workspace), _nbytes(workspace), _stream()))
    return x_out


def hyb_cfg_disc_euler_noalloc(v_c, v_u, x, x_out, scale, t, t_next, disc_l1=None, disc_l2=None, x_out_lowp=None,
                               v_out=None):
    batch = v_c.shape[0]
    n = v_c.numel() // batch if batch else 0
    _check(lib().hyb_cfg_disc_euler_noalloc(_p(v_c), _p(v_u, v_c.dtype), _p(x, torch.float32), _p(x_out, torch.float32),
                                            _p(x_out_lowp, torch.bfloat16), _p(v_out, v_c.dtype), batch, n, scale, t,
                                            t_next, _p(disc_l1, torch.float32), _p(disc_l2, torch.float32), _dt(v_c),
                                            _stream()))
    return x_out


def hyb_cfg_disc_affine(v_c, v_u, x, x_out, scale, a, b, disc_l1=None, disc_l2=None, workspace=None,
                        x_out_lowp=None, v_out=None):
    batch = v_c.shape[0]
    n = v_c.numel() // batch if batch else 0
    _check(lib().hyb_cfg_disc_affine(_p(v_c), _p(v_u, v_c.dtype), _p(x, torch.float32), _p(x_out, torch.float32),
                                     _p(x_out_lowp, torch.bfloat16), _p(v_out, v_c.dtype), batch, n, scale, a, b,
                                     _p(disc_l1, torch.float32), _p(disc_l2, torch.float32), _dt(v_c),
                                     _p(workspace), _nbytes(workspace), _stream()))
    return x_out


def hyb_joint_attention(q, k, v, o, scale=0.0):
    """q: [B, H, Nq, d]; k, v: [B, H, Nk, d]; o: [B, Nq, H*d]."""
    B, H, Nq, d = q.shape
    _check(lib().hyb_joint_attention(_p(q), _p(k, q.dtype), _p(v, q.dtype), _p(o, q.dtype), B, H, Nq, k.shape[2], d,
                                     scale, _dt(q), _stream()))
    return o


def hyb_joint_attention_workspace_bytes(batch, heads, n_q, dtype):
    return lib().hyb_joint_attention_workspace_bytes(batch, heads, n_q, dtype)


def hyb_joint_attention_ws(q, k, v, o, workspace, scale=0.0):
    """hyb_joint_attention with scratch (torch.uint8 tensor of hyb_joint_attention_workspace_bytes, or None)."""
    B, H, Nq, d = q.shape
    _check(lib().hyb_joint_attention_ws(_p(q), _p(k, q.dtype), _p(v, q.dtype), _p(o, q.dtype), B, H, Nq, k.shape[2], d,
                                        scale, _dt(q), _p(workspace), _nbytes(workspace), _stream()))
    return o


def hyb_joint_attention_prescaled(q, k, v, o, workspace):
    """hyb_joint_attention_ws for q that already holds q * scale * log2(e)."""
    B, H, Nq, d = q.shape
    _check(lib().hyb_joint_attention_prescaled(_p(q), _p(k, q.dtype), _p(v, q.dtype), _p(o, q.dtype), B, H, Nq, k.shape[2], d,
                                               _dt(q), _p(workspace), _nbytes(workspace), _stream()))
    return o


def hyb_adaln_modulation(w, bias, temb, out):
    """w: [rows, hidden]; bias: f32[rows]; temb: f32[batch, hidden]; out: f32[batch, rows]."""
    _check(lib().hyb_adaln_modulation(_p(w), _p(bias, torch.float32), _p(temb, torch.float32), _p(out, torch.float32),
                                      w.shape[0], w.shape[1], temb.shape[0], _dt(w), _stream()))
    return out


def hyb_layernorm_modulate(x, shift, scale, mod_stride, out, eps):
    """x: f32[B, T, D]; shift/scale: f32 views (first element of sample 0) or None; out: [B, T, D]."""
    B, T, D = x.shape
    ps = None if shift is None else C.c_void_p(shift.data_ptr())
    pc = None if scale is None else C.c_void_p(scale.data_ptr())
    _check(lib().hyb_layernorm_modulate(_p(x, torch.float32), ps, pc, mod_stride, _p(out), B, T, D, eps, _dt(out),
                                        _stream()))
    return out


def hyb_linear(a, w, bias, out, epi=HYB_EPI_BIAS, residual=None, gate=None, rows_per_gate=1, gate_stride=0):
    """a: [m, k]; w: [n, k] (HYB_EPI_GEGLU: [2n, k]); out: [m, n]."""
    m, k = a.shape
    n = out.shape[1]
    pg = None if gate is None else C.c_void_p(gate.data_ptr())
    _check(lib().hyb_linear(_p(a), _p(w, a.dtype), _p(bias, torch.float32), _p(out), m, n, k, _dt(a), _dt(out), epi,
                            _p(residual, torch.float32), pg, rows_per_gate, gate_stride, _stream()))
    return out


def block_desc(batch, n_img, n_txt, hidden, heads, dtype, head_dim=64, mlp_ratio=4, ln_eps=1e-6, txt_pre_only=False):
    return BlockDesc(batch, n_img, n_txt, hidden, heads, head_dim, mlp_ratio, dtype, ln_eps, int(txt_pre_only))


def block_weights(img, txt):
    """img / txt: dicts of tensors qkv_w, qkv_b, out_w, out_b, fc1_w, fc1_b, fc2_w, fc2_b."""
    def sw(d):
        return StreamWeights(*[d[n].data_ptr() for n in ("qkv_w", "out_w", "fc1_w", "fc2_w",
                                                          "qkv_b", "out_b", "fc1_b", "fc2_b")])
    return BlockWeights(sw(img), sw(txt))


def hyb_block_workspace_bytes(desc):
    return lib().hyb_block_workspace_bytes(C.byref(desc))


def hyb_block_forward(desc, weights, x_img_in, x_txt_in, mod_img, mod_txt, mod_stride, x_img_out, x_txt_out,
                      workspace):
    """mod_img / mod_txt: f32 views whose data_ptr is the first modulation value of sample 0."""
    _check(lib().hyb_block_forward(C.byref(desc), C.byref(weights), _p(x_img_in, torch.float32),
                                   _p(x_txt_in, torch.float32), C.c_void_p(mod_img.data_ptr()),
                                   C.c_void_p(mod_txt.data_ptr()), mod_stride, _p(x_img_out, torch.float32),
                                   _p(x_txt_out, torch.float32), _p(workspace), _nbytes(workspace), _stream()))


def hyb_timestep_embedding(t, out):
    _check(lib().hyb_timestep_embedding(_p(t, torch.float32), _p(out), out.shape[0], out.shape[1], _dt(out), _stream()))
    return out


def hyb_patchify(latent, tokens, p):
    B, Hh, Ww, Cc = latent.shape
    _check(lib().hyb_patchify(_p(latent, torch.float32), _p(tokens), B, Hh, Ww, Cc, p, _dt(tokens), _stream()))
    return tokens


def hyb_unpatchify(tokens, latent, p):
    B, Hh, Ww, Cc = latent.shape
    _check(lib().hyb_unpatchify(_p(tokens), _p(latent), B, Hh, Ww, Cc, p, _dt(tokens), _dt(latent), _stream()))
    return latent


def hyb_convert(src, out):
    _check(lib().hyb_convert(_p(src, torch.float32), _p(out), src.numel(), _dt(out), _stream()))
    return out


def hyb_trace_enable(on):
    _check(lib().hyb_trace_enable(1 if on else 0))


def hyb_trace_summary():
    """-> {kernel name: {"unit", "launches", "ms", "work"}} for the launches recorded since tracing was enabled."""
    buf = C.create_string_buffer(1 << 16)
    _check(lib().hyb_trace_summary(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, unit, count, ms, work = line.split("\t")
        out[name] = {"unit": unit, "launches": int(count), "ms": float(ms), "work": float(work)}
    return out


def hyb_groupnorm_workspace_bytes(batch, groups):
    return lib().hyb_groupnorm_workspace_bytes(batch, groups)


def hyb_groupnorm(x, gamma, beta, out, groups, eps, workspace):
    """x, out: f32[B, T, C]."""
    B, T, Cc = x.shape
    _check(lib().hyb_groupnorm(_p(x, torch.float32), _p(gamma, torch.float32), _p(beta, torch.float32),
                               _p(out, torch.float32), B, T, Cc, groups, eps, _p(workspace), _nbytes(workspace), _stream()))
    return out


def hyb_layernorm_affine(x, gamma, beta, out, eps):
    """x: f32[..., hidden]; out: same shape."""
    hidden = x.shape[-1]
    _check(lib().hyb_layernorm_affine(_p(x, torch.float32), _p(gamma, torch.float32), _p(beta, torch.float32), _p(out),
                                      x.numel() // hidden, hidden, eps, _dt(out), _stream()))
    return out


def sdxl_block_desc(batch, tokens, channels, heads, n_ctx, ctx_dim, dtype, groups=32, gn_eps=1e-5, ln_eps=1e-5):
    return SdxlBlockDesc(batch, tokens, channels, heads, 64, n_ctx, ctx_dim, groups, dtype, gn_eps, ln_eps)


def sdxl_block_weights(d):
    """d: dict of device tensors named as the fields of hyb_sdxl_block_weights."""
    return SdxlBlockWeights(*[d[n].data_ptr() for n in SDXL_WEIGHT_FIELDS])


def hyb_sdxl_block_workspace_bytes(desc):
    return lib().hyb_sdxl_block_workspace_bytes(C.byref(desc))


def hyb_sdxl_block_forward(desc, weights, x_in, ctx, x_out, workspace):
    _check(lib().hyb_sdxl_block_forward(C.byref(desc), C.byref(weights), _p(x_in, torch.float32), _p(ctx),
                                        _p(x_out, torch.float32), _p(workspace), _nbytes(workspace), _stream()))
    return x_out


def hyb_switch_init(total_steps, window, g_slope, tau_cap, k):
    st = SwitchState()
    _check(lib().hyb_switch_init(C.byref(st), total_steps, window, g_slope, tau_cap, k))
    return st


def hyb_switch_push(state, discrepancy):
    stage = C.c_int(-1)
    _check(lib().hyb_switch_push(C.byref(state), discrepancy, C.byref(stage)))
    return stage.value


def hyb_switch_stage(state, step):
    return lib().hyb_switch_stage(C.byref(state), step)
