"""Argument marshalling for the C ABI of include/sama.h.  No arithmetic of the method happens here: torch
supplies device memory and the current HIP stream, every step runs in the library's kernels.  There is no CPU
fallback: without libsama.so (or without a GPU) construction fails."""
import ctypes as C
import os

MODEL_MLP, MODEL_ENCODER = 0, 1
DTYPE_FP32, DTYPE_BF16 = 0, 1
OPT_SGD, OPT_ADAM = 0, 1
ADAPT_OPTIMIZER, ADAPT_NONE = 0, 1
STATE = dict(THETA=0, LAMBDA=1, M=2, V=3, G=4, GMETA=5, VDIR=6, META_M=7, META_V=8, COUNTERS=9, HYPERGRAD=10,
             GLAM_PLUS=11, GLAM_MINUS=12, SCALARS=13, LOSSES=14)


class SamaConfig(C.Structure):
    _fields_ = [("model_kind", C.c_int32), ("n_dims", C.c_int32), ("dims", C.c_int32 * 8),
                ("param_dtype", C.c_int32), ("wnet_hidden", C.c_int32), ("base_opt", C.c_int32),
                ("base_lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("weight_decay", C.c_float), ("momentum", C.c_float), ("meta_lr", C.c_float), ("meta_beta1", C.c_float),
                ("meta_beta2", C.c_float), ("meta_eps", C.c_float), ("alpha", C.c_float),
                ("adapt_mode", C.c_int32), ("max_batch", C.c_int32), ("max_meta_batch", C.c_int32),
                ("fast_meta_pass", C.c_int32), ("fast_base_pass", C.c_int32), ("corr_hidden", C.c_int32), ("corr_kappa", C.c_float),
                ("aux_mlm", C.c_int32), ("max_aux_batch", C.c_int32), ("max_aux_masked", C.c_int32)]

    @classmethod
    def make(cls, kind, dims, *, H, max_batch, max_meta_batch, base_opt=OPT_ADAM, base_lr=1e-3, beta1=0.9,
             beta2=0.999, adam_eps=1e-8, weight_decay=0.0, meta_lr=1e-3, meta_beta1=0.9, meta_beta2=0.999,
             meta_eps=1e-8, alpha=1.0, adapt_mode=ADAPT_OPTIMIZER, bf16=None, fast_meta_pass=0, fast_base_pass=0, momentum=0.0, corr_hidden=0,
             corr_kappa=4.0, aux_mlm=0, max_aux_batch=0, max_aux_masked=0):
        c = cls()
        c.model_kind = MODEL_MLP if kind == "mlp" else MODEL_ENCODER
        c.n_dims = len(dims)
        for i, d in enumerate(dims):
            c.dims[i] = int(d)
        if bf16 is None:
            bf16 = kind == "encoder"
        c.param_dtype = DTYPE_BF16 if bf16 else DTYPE_FP32
        c.wnet_hidden = H
        c.base_opt, c.base_lr, c.beta1, c.beta2, c.adam_eps, c.weight_decay = base_opt, base_lr, beta1, beta2, adam_eps, weight_decay
        c.meta_lr, c.meta_beta1, c.meta_beta2, c.meta_eps = meta_lr, meta_beta1, meta_beta2, meta_eps
        c.alpha, c.adapt_mode, c.max_batch, c.max_meta_batch = alpha, adapt_mode, max_batch, max_meta_batch
        c.fast_meta_pass, c.fast_base_pass, c.momentum = fast_meta_pass, fast_base_pass, momentum
        c.corr_hidden, c.corr_kappa = corr_hidden, corr_kappa
        c.aux_mlm, c.max_aux_batch, c.max_aux_masked = aux_mlm, max_aux_batch, max_aux_masked
        return c


class SamaBatch(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("sample_mask", C.c_void_p), ("n", C.c_int32), ("seq_len", C.c_void_p)]


class SamaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libsama error {code}: {msg}")
        self.code = code


def lib_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsama.so")


class SamaAuxBatch(C.Structure):
    _fields_ = [("ids", C.c_void_p), ("mask_row", C.c_void_p), ("mask_tgt", C.c_void_p), ("n_seq", C.c_int32), ("n_mask", C.c_int32),
                ("seq_len", C.c_void_p)]


_lib = None


def load_library():
    """dlopen the in-tree libsama.so and declare the prototypes of include/sama.h.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    p = lib_path()
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(p)
    cfgp = C.POINTER(SamaConfig)
    L.sama_param_count.restype = C.c_int64; L.sama_param_count.argtypes = [cfgp]
    L.sama_gemm_param_count.restype = C.c_int64; L.sama_gemm_param_count.argtypes = [cfgp]
    L.sama_lambda_count.restype = C.c_int32; L.sama_lambda_count.argtypes = [cfgp]
    L.sama_param_tensor_count.restype = C.c_int32; L.sama_param_tensor_count.argtypes = [cfgp]
    L.sama_param_tensor.restype = C.c_int; L.sama_param_tensor.argtypes = [cfgp, C.c_int32, C.c_char_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.sama_workspace_bytes.restype = C.c_size_t; L.sama_workspace_bytes.argtypes = [cfgp]
    L.sama_init.restype = C.c_int; L.sama_init.argtypes = [cfgp, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
    bp = C.POINTER(SamaBatch)
    L.sama_base_step.restype = C.c_int; L.sama_base_step.argtypes = [C.c_void_p, bp, C.c_void_p]
    L.sama_meta_grad.restype = C.c_int; L.sama_meta_grad.argtypes = [C.c_void_p, bp, bp, C.c_void_p, C.c_void_p]
    L.sama_meta_step.restype = C.c_int; L.sama_meta_step.argtypes = [C.c_void_p, bp, bp]
    ap = C.POINTER(SamaAuxBatch)
    L.sama_aux_base_step.restype = C.c_int; L.sama_aux_base_step.argtypes = [C.c_void_p, bp, ap, C.c_void_p]
    L.sama_aux_meta_grad.restype = C.c_int; L.sama_aux_meta_grad.argtypes = [C.c_void_p, ap, bp, C.c_void_p, C.c_void_p]
    L.sama_aux_meta_step.restype = C.c_int; L.sama_aux_meta_step.argtypes = [C.c_void_p, ap, bp]
    L.sama_get_state.restype = C.c_int; L.sama_get_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    L.sama_set_state.restype = C.c_int; L.sama_set_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    L.sama_profile_family_count.restype = C.c_int32; L.sama_profile_family_count.argtypes = []
    L.sama_profile_enable.restype = C.c_int; L.sama_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    L.sama_profile_read.restype = C.c_int; L.sama_profile_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.sama_last_error.restype = C.c_char_p; L.sama_last_error.argtypes = [C.c_void_p]
    L.sama_destroy.restype = None; L.sama_destroy.argtypes = [C.c_void_p]
    vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_float
    L.sama_op_gemm_bf16.restype = C.c_int
    L.sama_op_gemm_bf16.argtypes = [vp, i64, i32, vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, i64, vp]
    L.sama_op_gemm_bf16_batch.restype = C.c_int
    L.sama_op_gemm_bf16_batch.argtypes = [i32, vp, vp, vp, vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), i32, i32, vp]
    L.sama_set_lr.restype = C.c_int; L.sama_set_lr.argtypes = [vp, f32, f32]
    L.sama_eval.restype = C.c_int; L.sama_eval.argtypes = [vp, vp, vp, vp, vp]
    L.sama_aux_eval.restype = C.c_int; L.sama_aux_eval.argtypes = [vp, vp, vp, vp]
    L.sama_op_adam.restype = C.c_int
    L.sama_op_adam.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, f32, f32, f32, f32, vp]
    L.sama_op_adapt_norm.restype = C.c_int
    L.sama_op_adapt_norm.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, f32, f32, f32, f32, f32, vp, vp, vp]
    L.sama_op_adapt_norm_static.restype = C.c_int
    L.sama_op_adapt_norm_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, f32, f32, f32, f32, f32, vp, vp, vp]
    L.sama_op_last_error.restype = C.c_char_p; L.sama_op_last_error.argtypes = []
    L.sama_op_perturb_lo.restype = C.c_int; L.sama_op_perturb_lo.argtypes = [vp, vp, vp, vp, vp, i64, vp]
    L.sama_op_nudge.restype = C.c_int; L.sama_op_nudge.argtypes = [vp, vp, vp, vp, i64, i64, vp]
    _lib = L
    return L


def param_tensors(cfg):
    """[(name, offset, rows, cols)] as the library lays theta out."""
    L = load_library()
    out = []
    for i in range(L.sama_param_tensor_count(C.byref(cfg))):
        name = C.create_string_buffer(32)
        off, r, c = C.c_int64(), C.c_int64(), C.c_int64()
        rc = L.sama_param_tensor(C.byref(cfg), i, name, C.byref(off), C.byref(r), C.byref(c))
        if rc != 0:
            raise SamaError(rc, L.sama_last_error(None).decode())
        out.append((name.value.decode(), off.value, r.value, c.value))
    return out


class Sama:
    """One SAMA context on the current CUDA(HIP) device and torch's current stream."""

    def __init__(self, cfg, theta0, lambda0):
        import torch
        self.torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("libsama needs a GPU: there is no CPU path")
        self.cfg = cfg
        self.n = self.lib.sama_param_count(C.byref(cfg))
        self.nl = self.lib.sama_lambda_count(C.byref(cfg))
        nbytes = self.lib.sama_workspace_bytes(C.byref(cfg))
        if self.n < 0 or nbytes == 0:
            raise SamaError(1, self.lib.sama_last_error(None).decode())
        self.dev = torch.device("cuda", torch.cuda.current_device())
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        th = self._dev_f32(theta0, self.n)
        lam = self._dev_f32(lambda0, self.nl)
        self.stream = torch.cuda.current_stream(self.dev)
        h = C.c_void_p()
        rc = self.lib.sama_init(C.byref(cfg), base, nbytes, th.data_ptr(), lam.data_ptr(), self.stream.cuda_stream, C.byref(h))
        if rc != 0:
            raise SamaError(rc, self.lib.sama_last_error(None).decode())
        self.h = h
        self._keep = [th, lam]
        self.max_b = max(cfg.max_batch + (cfg.max_aux_batch if cfg.aux_mlm else 0), cfg.max_meta_batch)

    def _dev_f32(self, a, count):
        torch = self.torch
        t = a if isinstance(a, torch.Tensor) else torch.as_tensor(a)
        t = t.to(device=self.dev, dtype=torch.float32).contiguous()
        if t.numel() != count:
            raise ValueError(f"expected {count} elements, got {t.numel()}")
        return t

    def _check(self, rc):
        if rc != 0:
            raise SamaError(rc, self.lib.sama_last_error(self.h).decode())

    def batch(self, x, y, mask=None, seq_len=None):
        """Device tensors (x fp32 [n, d0] or int32 [n, S]; y int32 [n]; mask uint8 [n] or None; seq_len int32 [n] or
        None) -> sama_batch."""
        torch = self.torch
        assert x.is_cuda and y.is_cuda and x.is_contiguous() and y.dtype == torch.int32
        assert x.dtype in (torch.float32, torch.int32)
        if seq_len is not None:
            assert seq_len.is_cuda and seq_len.is_contiguous() and seq_len.dtype == torch.int32 and seq_len.numel() == y.numel()
        b = SamaBatch(x.data_ptr(), y.data_ptr(), None if mask is None else mask.data_ptr(), int(y.numel()),
                      None if seq_len is None else seq_len.data_ptr())
        b._keep = (x, y, mask, seq_len)
        if mask is not None:
            assert mask.dtype == torch.uint8 and mask.is_cuda and mask.numel() == y.numel()
        return b

    def base_step(self, train, loss_out=None):
        self._check(self.lib.sama_base_step(self.h, C.byref(train), None if loss_out is None else loss_out.data_ptr()))

    def meta_grad(self, train, meta, hypergrad_out=None, eps_out=None):
        self._check(self.lib.sama_meta_grad(self.h, C.byref(train), C.byref(meta),
                                            None if hypergrad_out is None else hypergrad_out.data_ptr(),
                                            None if eps_out is None else eps_out.data_ptr()))

    def meta_step(self, train, meta):
        self._check(self.lib.sama_meta_step(self.h, C.byref(train), C.byref(meta)))

    def eval(self, batch, logits_out=None, losses_out=None, weights_out=None):
        """Forward only: fp32 device tensors logits_out [n, C], losses_out [n], weights_out [n], each optional."""
        p = lambda t: None if t is None else t.data_ptr()
        for t in (logits_out, losses_out, weights_out):
            assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == self.torch.float32)
        self._check(self.lib.sama_eval(self.h, C.byref(batch), p(logits_out), p(losses_out), p(weights_out)))

    def aux_eval(self, pt, losses_out=None, weights_out=None):
        p = lambda t: None if t is None else t.data_ptr()
        for t in (losses_out, weights_out):
            assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == self.torch.float32)
        self._check(self.lib.sama_aux_eval(self.h, C.byref(pt), p(losses_out), p(weights_out)))

    def set_lr(self, base_lr, meta_lr):
        self._check(self.lib.sama_set_lr(self.h, base_lr, meta_lr))

    def aux_batch(self, ids, mask_row, mask_tgt, seq_len=None):
        """Device int32 tensors (ids [n_seq, S], mask_row [n_mask] = sequence * S + position, mask_tgt [n_mask], seq_len
        [n_seq] or None) -> sama_aux_batch."""
        torch = self.torch
        for t in (ids, mask_row, mask_tgt) + (() if seq_len is None else (seq_len,)):
            assert t.is_cuda and t.is_contiguous() and t.dtype == torch.int32
        assert mask_row.numel() == mask_tgt.numel() and (seq_len is None or seq_len.numel() == ids.shape[0])
        b = SamaAuxBatch(ids.data_ptr(), mask_row.data_ptr(), mask_tgt.data_ptr(), int(ids.shape[0]), int(mask_row.numel()),
                         None if seq_len is None else seq_len.data_ptr())
        b._keep = (ids, mask_row, mask_tgt, seq_len)
        return b

    def aux_base_step(self, ft, pt, loss_out=None):
        self._check(self.lib.sama_aux_base_step(self.h, C.byref(ft), C.byref(pt), None if loss_out is None else loss_out.data_ptr()))

    def aux_meta_grad(self, pt, meta, hypergrad_out=None, eps_out=None):
        self._check(self.lib.sama_aux_meta_grad(self.h, C.byref(pt), C.byref(meta),
                                                None if hypergrad_out is None else hypergrad_out.data_ptr(),
                                                None if eps_out is None else eps_out.data_ptr()))

    def aux_meta_step(self, pt, meta):
        self._check(self.lib.sama_aux_meta_step(self.h, C.byref(pt), C.byref(meta)))

    def get_state(self, name):
        torch = self.torch
        which = STATE[name]
        if name == "COUNTERS":
            out = torch.empty(4, dtype=torch.int64, device=self.dev)
        elif name == "SCALARS":
            out = torch.empty(4, dtype=torch.float32, device=self.dev)
        elif name == "LOSSES":
            out = torch.empty(self.max_b, dtype=torch.float32, device=self.dev)
        elif name in ("LAMBDA", "META_M", "META_V", "HYPERGRAD", "GLAM_PLUS", "GLAM_MINUS"):
            out = torch.empty(self.nl, dtype=torch.float32, device=self.dev)
        else:
            out = torch.empty(self.n, dtype=torch.float32, device=self.dev)
        self._check(self.lib.sama_get_state(self.h, which, out.data_ptr()))
        return out

    def set_state(self, name, value):
        torch = self.torch
        if name == "COUNTERS":
            t = torch.as_tensor(value).to(device=self.dev, dtype=torch.int64).contiguous()
            assert t.numel() == 4
        else:
            t = self._dev_f32(value, self.nl if name in ("LAMBDA", "META_M", "META_V") else self.n)
        self._check(self.lib.sama_set_state(self.h, STATE[name], t.data_ptr()))
        self.stream.synchronize()      # `t` may be freed once we return

    def profile(self, on):
        self._check(self.lib.sama_profile_enable(self.h, 1 if on else 0))

    def profile_read(self):
        """{family name: (launches, total_ms, units)} for every family with at least one launch."""
        out = {}
        for f in range(self.lib.sama_profile_family_count()):
            name, n, ms, u = C.c_char_p(), C.c_int64(), C.c_double(), C.c_double()
            self._check(self.lib.sama_profile_read(self.h, f, C.byref(name), C.byref(n), C.byref(ms), C.byref(u)))
            if n.value:
                out[name.value.decode()] = (n.value, ms.value, u.value)
        return out

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.dev)
            self.lib.sama_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------------------------------------- op-level calls
def _p(t):
    return None if t is None else t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def op_gemm_bf16(A, B, *, a_trans=False, b_trans=True, B2=None, bias=None, out32=None, out16=None):
    """C = A . (B + B2) (+ bias) through sama_op_gemm_bf16.  A, B, B2: 2-D contiguous torch.bfloat16 CUDA tensors in
    the storage the flags describe; out32 / out16: preallocated [M, N] outputs."""
    L = load_library()
    K, M = (A.shape[0], A.shape[1]) if a_trans else (A.shape[1], A.shape[0])
    N = B.shape[0] if b_trans else B.shape[1]
    out = out32 if out32 is not None else out16
    rc = L.sama_op_gemm_bf16(_p(A), A.stride(0), int(a_trans), _p(B), _p(B2), B.stride(0), int(b_trans), M, N, K, _p(bias),
                             _p(out32), _p(out16), out.stride(0), _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_gemm_bf16 rejected the arguments")


def op_gemm_bf16_batch(As, Bs, outs, *, a_trans=False, b_trans=True, B2s=None):
    """Several independent C_k = A_k . (B_k + B2_k) in one launch through sama_op_gemm_bf16_batch (dense 2-D bf16 operands,
    fp32 outputs)."""
    L = load_library()
    n = len(As)
    Ms, Ns, Ks = [], [], []
    for A, B in zip(As, Bs):
        K, M = (A.shape[0], A.shape[1]) if a_trans else (A.shape[1], A.shape[0])
        Ms.append(M); Ks.append(K); Ns.append(B.shape[0] if b_trans else B.shape[1])
    vp = C.c_void_p * n
    ia = C.c_int32 * n
    rc = L.sama_op_gemm_bf16_batch(n, vp(*[A.data_ptr() for A in As]), vp(*[B.data_ptr() for B in Bs]),
                                   vp(*[b.data_ptr() for b in B2s]) if B2s is not None else None,
                                   vp(*[o.data_ptr() for o in outs]), ia(*Ms), ia(*Ns), ia(*Ks), int(a_trans), int(b_trans), _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_gemm_bf16_batch rejected the arguments")


def op_adam(g, m, v, theta, theta16, n16, t, lr, beta1, beta2, eps, wd=0.0):
    rc = load_library().sama_op_adam(_p(g), _p(m), _p(v), _p(theta), _p(theta16), theta.numel(), n16, t, lr, beta1, beta2, eps, wd, _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_adam rejected the arguments")


def op_adapt_norm(g, m, v, gmeta, vdir, partial, t, lr, beta1, beta2, eps, alpha, scalars, status):
    rc = load_library().sama_op_adapt_norm(_p(g), _p(m), _p(v), _p(gmeta), _p(vdir), _p(partial), g.numel(), t, lr, beta1, beta2,
                                           eps, alpha, _p(scalars), _p(status), _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_adapt_norm rejected the arguments")


def op_adapt_norm_static(g, m, v, gmeta, vdir, t, lr, beta1, beta2, eps, alpha, scalars, status, n=None):
    """sama_op_adapt_norm with the library's own static scratch (allocates nothing); n defaults to g.numel()."""
    L = load_library()
    rc = L.sama_op_adapt_norm_static(_p(g), _p(m), _p(v), _p(gmeta), _p(vdir), g.numel() if n is None else n, t, lr, beta1, beta2,
                                     eps, alpha, _p(scalars), _p(status), _stream())
    if rc != 0:
        raise SamaError(rc, L.sama_op_last_error().decode() or "sama_op_adapt_norm_static failed")


def op_perturb_lo(theta, vdir, eps_t, lo_p, lo_m, n16):
    rc = load_library().sama_op_perturb_lo(_p(theta), _p(vdir), _p(eps_t), _p(lo_p), _p(lo_m), n16, _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_perturb_lo rejected the arguments")


def op_nudge(theta, vdir, eps_t, theta16, n16):
    rc = load_library().sama_op_nudge(_p(theta), _p(vdir), _p(eps_t), _p(theta16), theta.numel(), n16, _stream())
    if rc != 0:
        raise SamaError(rc, "sama_op_nudge rejected the arguments")
