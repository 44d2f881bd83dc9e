"""Shared plumbing of the GPU parity tests: build the oracle and the HIP context from one workload, move
oracle state INTO the GPU context (never the other way), compare with relative L2 error."""
import numpy as np


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def make_pair(wl, theta0, lambda0, **over):
    """(oracle, gpu context) with identical hyper-parameters."""
    import torch
    import paper_2310_05674_amd as pkg
    from oracle import models
    from oracle.reweight import SamaOracle, ADAM, SGD
    kw = dict(base_lr=wl.base_lr, meta_lr=wl.meta_lr, alpha=wl.alpha, beta1=wl.beta1, beta2=wl.beta2,
              adam_eps=wl.adam_eps)
    kw.update({k: v for k, v in over.items() if k in ("base_lr", "meta_lr", "alpha", "adam_eps", "weight_decay", "momentum")})
    base_opt = over.get("base_opt", "adam")
    adapt = over.get("adapt_mode", 0)
    corr = {k: over[k] for k in ("corr_hidden", "corr_kappa") if k in over}
    gpu_only = {k: over[k] for k in ("fast_base_pass", "fast_meta_pass") if k in over}   # precision switches of the HIP path
    orc = SamaOracle(models.make_model(wl.kind, wl.dims), theta0, lambda0, base_opt=ADAM if base_opt == "adam" else SGD,
                     adapt_mode=adapt, n_classes=wl.dims[-1] if corr.get("corr_hidden") else None, **corr, **kw)
    cfg = pkg.SamaConfig.make(wl.kind, wl.dims, H=wl.H, max_batch=over.get("max_batch", wl.batch),
                              max_meta_batch=over.get("max_meta_batch", wl.meta_batch),
                              base_opt=pkg.OPT_ADAM if base_opt == "adam" else pkg.OPT_SGD, adapt_mode=adapt, **corr, **gpu_only, **kw)
    gpu = pkg.Sama(cfg, theta0, lambda0)
    return orc, gpu


def make_aux_pair(wl, theta0, lambda0, max_aux_batch, max_aux_masked, **over):
    """(AuxTaskOracle, gpu context) for an encoder workload with the masked-token head (wl.mlm must be set)."""
    import paper_2310_05674_amd as pkg
    from oracle import models
    from oracle.auxtask import AuxTaskOracle
    kw = dict(base_lr=wl.base_lr, meta_lr=wl.meta_lr, alpha=wl.alpha, beta1=wl.beta1, beta2=wl.beta2,
              adam_eps=wl.adam_eps)
    kw.update({k: v for k, v in over.items() if k in ("base_lr", "meta_lr", "alpha", "adam_eps", "weight_decay")})
    orc = AuxTaskOracle(models.make_model(wl.kind, wl.dims, mlm=True), theta0, lambda0, **kw)
    cfg = pkg.SamaConfig.make(wl.kind, wl.dims, H=wl.H, max_batch=wl.batch, max_meta_batch=wl.meta_batch, aux_mlm=1,
                              max_aux_batch=max_aux_batch, max_aux_masked=max_aux_masked, **kw)
    return orc, pkg.Sama(cfg, theta0, lambda0)


def dev_aux_batch(gpu, ids, seq, pos, tgt, lens=None):
    import torch
    S = ids.shape[1]
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a).astype(np.int32), device=gpu.dev)
    return gpu.aux_batch(t(ids), t(seq.astype(np.int64) * S + pos), t(tgt), None if lens is None else t(lens))


def dev_batch(gpu, x, y, mask=None, lens=None):
    import torch
    xt = torch.as_tensor(np.ascontiguousarray(x), device=gpu.dev)
    yt = torch.as_tensor(np.ascontiguousarray(y).astype(np.int32), device=gpu.dev)
    mt = None if mask is None else torch.as_tensor(np.ascontiguousarray(mask).astype(np.uint8), device=gpu.dev)
    lt = None if lens is None else torch.as_tensor(np.ascontiguousarray(lens).astype(np.int32), device=gpu.dev)
    return gpu.batch(xt, yt, mt, lt)


def push_state(orc, gpu):
    """Teacher forcing: the oracle's state, rounded to fp32, becomes the GPU context's state."""
    for name, arr in (("THETA", orc.theta), ("M", orc.m), ("V", orc.v), ("G", orc.g), ("LAMBDA", orc.lam),
                      ("META_M", orc.meta_m), ("META_V", orc.meta_v)):
        gpu.set_state(name, arr.astype(np.float32))
    gpu.set_state("COUNTERS", np.array([orc.t, orc.meta_t, 0, 0], dtype=np.int64))


def pull(gpu, name):
    return gpu.get_state(name).cpu().numpy()
