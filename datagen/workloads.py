"""Synthetic stand-ins for the paper's noisy-label data-reweighting runs (Sec. 4.1, Table 4).

Five workloads, numbered 1..5 as in the benchmark's `configs`.  Everything is drawn from
CounterRNG(seed = 20231005 + config id) on fixed stream numbers, so a data set is a pure
function of its config id.  Nothing here evaluates a loss, a gradient or an optimizer.
"""
from dataclasses import dataclass, field
import numpy as np
from .rng import CounterRNG

BASE_SEED = 20231005

# stream numbers (one namespace per workload seed)
S_X, S_TEACHER, S_FLIP_PERM, S_FLIP_LABEL, S_XMETA, S_MEANS, S_CLASS, S_CLASS_META = 1, 2, 3, 4, 5, 6, 7, 8
S_TOK, S_TOK_META, S_THETA, S_LAMBDA, S_LAMBDA_CORR, S_EPOCH_PERM = 9, 10, 11, 12, 13, 1000
S_TOK_AUX, S_AUX_COUNT, S_AUX_PERM = 14, 15, 2000000
S_LENGTHS = 16


@dataclass
class Workload:
    cfg: int
    kind: str                      # "mlp" | "encoder"
    dims: tuple                    # mlp: layer widths; encoder: (L, d, heads, ffn, S, V, C)
    bf16: bool
    H: int                         # weight-net hidden width
    batch: int
    meta_batch: int
    base_lr: float
    meta_lr: float
    alpha: float
    noise: float
    n_train: int
    n_meta: int
    steps: int
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    mlm: bool = False              # encoder with a masked-token head (auxiliary-task reweighting)
    # filled by make_workload
    x_train: np.ndarray = field(default=None, repr=False)
    y_train: np.ndarray = field(default=None, repr=False)      # noisy labels (int32)
    y_train_clean: np.ndarray = field(default=None, repr=False)
    flipped: np.ndarray = field(default=None, repr=False)      # bool mask of flipped labels
    x_meta: np.ndarray = field(default=None, repr=False)
    y_meta: np.ndarray = field(default=None, repr=False)

    @property
    def seed(self):
        return BASE_SEED + self.cfg

    @property
    def n_classes(self):
        return self.dims[-1]

    def train_batch(self, step):
        """Indices of the train batch of base step `step` (0-based): sequential slices of a
        per-epoch permutation (full batch for cfg 1)."""
        return _batch(self.seed, S_EPOCH_PERM, self.n_train, self.batch, step)

    def meta_batch_idx(self, step):
        return _batch(self.seed, S_EPOCH_PERM + 500000, self.n_meta, self.meta_batch, step)


def _batch(seed, stream0, n, b, step):
    if b >= n:
        return np.arange(n, dtype=np.int64)
    per_epoch = n // b
    epoch, k = divmod(step, per_epoch)
    perm = CounterRNG(seed).permutation(stream0 + epoch, n)
    return perm[k * b:(k + 1) * b]


WORKLOADS = {
    1: dict(kind="mlp", dims=(32, 2), bf16=False, H=16, batch=512, meta_batch=64, base_lr=1e-2,
            meta_lr=1e-3, alpha=1e-2, noise=0.30, n_train=512, n_meta=64, steps=20),
    2: dict(kind="mlp", dims=(784, 256, 256, 10), bf16=False, H=100, batch=128, meta_batch=128,
            base_lr=1e-3, meta_lr=1e-3, alpha=1.0, noise=0.40, n_train=12800, n_meta=1280, steps=500),
    3: dict(kind="encoder", dims=(4, 256, 4, 1024, 128, 8192, 4), bf16=True, H=100, batch=32,
            meta_batch=32, base_lr=1e-5, meta_lr=1e-5, alpha=1.0, noise=0.30, n_train=4096,
            n_meta=512, steps=50),
    4: dict(kind="encoder", dims=(12, 768, 12, 3072, 128, 30522, 6), bf16=True, H=100, batch=32,
            meta_batch=32, base_lr=1e-5, meta_lr=1e-5, alpha=1.0, noise=0.20, n_train=4096,
            n_meta=512, steps=50),
    5: dict(kind="encoder", dims=(24, 1024, 16, 4096, 128, 50265, 2), bf16=True, H=100, batch=16,
            meta_batch=16, base_lr=1e-5, meta_lr=1e-5, alpha=1.0, noise=0.20, n_train=4096,
            n_meta=512, steps=50),
}


# ----------------------------------------------------------------------------- parameters
def param_layout(kind, dims, mlm=False):
    """Flat layout of theta: list of (name, shape, offset).  Rule: every GEMM weight matrix
    (stored [out x in], row-major) in layer order first, then every remaining tensor in layer
    order.  mlm: the encoder carries a masked-token head, its decoder Wmlm [V x d] last among
    the GEMM matrices and its bias bmlm [V] just before the classifier head (Wc, bc).  This restates the interface documented in include/sama.h; the oracle and the HIP
    library each hold their own statement of it and tests compare the three."""
    mats, vecs = [], []
    if kind == "mlp":
        for l in range(len(dims) - 1):
            mats.append((f"W{l}", (dims[l + 1], dims[l])))
            vecs.append((f"b{l}", (dims[l + 1],)))
    elif kind == "encoder":
        L, d, heads, ffn, S, V, C = dims
        for l in range(L):
            mats += [(f"l{l}.Wqkv", (3 * d, d)), (f"l{l}.Wo", (d, d)),
                     (f"l{l}.W1", (ffn, d)), (f"l{l}.W2", (d, ffn))]
            vecs += [(f"l{l}.bqkv", (3 * d,)), (f"l{l}.bo", (d,)), (f"l{l}.ln1_g", (d,)),
                     (f"l{l}.ln1_b", (d,)), (f"l{l}.b1", (ffn,)), (f"l{l}.b2", (d,)),
                     (f"l{l}.ln2_g", (d,)), (f"l{l}.ln2_b", (d,))]
        vecs += [("tok_emb", (V, d)), ("pos_emb", (S, d)), ("emb_ln_g", (d,)), ("emb_ln_b", (d,))]
        if mlm:
            mats.append(("Wmlm", (V, d)))
            vecs.append(("bmlm", (V,)))
        vecs += [("Wc", (C, d)), ("bc", (C,))]
    else:
        raise ValueError(kind)
    out, off = [], 0
    for name, shape in mats + vecs:
        out.append((name, shape, off))
        off += int(np.prod(shape))
    return out


def param_count(kind, dims, mlm=False):
    name, shape, off = param_layout(kind, dims, mlm)[-1]
    return off + int(np.prod(shape))


def round_to_bf16(a):
    """Round float values to the nearest bf16-representable value (ties to even), returned in
    the input's float64/float32 dtype.  Input preparation only."""
    f = np.asarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).astype(np.asarray(a).dtype).reshape(np.shape(a))


def init_theta(wl, scale=0.02):
    """Initial base parameters (float64 array holding float32- or bf16-representable values).
    `scale` is the std of the encoder's matrices and embeddings."""
    rng = CounterRNG(wl.seed)
    lay = param_layout(wl.kind, wl.dims, wl.mlm)
    n = param_count(wl.kind, wl.dims, wl.mlm)
    z = rng.normal(S_THETA, n)
    th = np.zeros(n, dtype=np.float64)
    for name, shape, off in lay:
        size = int(np.prod(shape))
        leaf = name.split(".")[-1]
        if wl.kind == "mlp":
            if leaf.startswith("W"):
                th[off:off + size] = z[off:off + size] / np.sqrt(shape[1])
        else:
            if leaf in ("ln1_g", "ln2_g", "emb_ln_g"):
                th[off:off + size] = 1.0
            elif leaf.startswith("W") or leaf.endswith("emb"):
                th[off:off + size] = scale * z[off:off + size]
    th = th.astype(np.float32).astype(np.float64)
    return round_to_bf16(th) if wl.bf16 else th


def init_lambda(wl):
    """Weight-net parameters, flat [W1(H), b1(H), W2(H), b2(1)], float32-representable."""
    H = wl.H
    z = CounterRNG(wl.seed).normal(S_LAMBDA, 3 * H + 1)
    lam = np.concatenate([z[:H], z[H:2 * H], z[2 * H:3 * H] / np.sqrt(H), [0.0]])
    return lam.astype(np.float32).astype(np.float64)


def init_lambda_corr(wl, corr_hidden):
    """Label-corrector parameters, flat [W1(Hc x 2C), b1(Hc), W2(C x Hc), b2(C)], float32-representable: small
    random weights, first-layer biases positive so that most hidden units start active."""
    C, Hc = wl.dims[-1], corr_hidden
    n1, n2 = Hc * 2 * C, C * Hc
    z = CounterRNG(wl.seed).normal(S_LAMBDA_CORR, n1 + Hc + n2 + C)
    lam = np.concatenate([z[:n1] / np.sqrt(2 * C), 0.25 + 0.25 * np.abs(z[n1:n1 + Hc]),
                          z[n1 + Hc:n1 + Hc + n2] / np.sqrt(Hc), 0.1 * z[n1 + Hc + n2:]])
    return lam.astype(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- data
def flip_labels(rng, y, n_classes, frac):
    """Flip exactly floor(frac*N) labels: the first entries of a seeded permutation get a new
    label uniform over the other C-1 classes."""
    n = len(y)
    k = int(np.floor(frac * n))
    perm = rng.permutation(S_FLIP_PERM, n)
    shift = 1 + rng.integers(S_FLIP_LABEL, n, n_classes - 1)     # in [1, C-1]
    y2 = y.copy()
    sel = perm[:k]
    y2[sel] = (y[sel] + shift[sel]) % n_classes
    flipped = np.zeros(n, dtype=bool)
    flipped[sel] = True
    return y2, flipped


def _zipf_tokens(rng, stream, n_seq, S, V, a=1.1):
    ranks = np.arange(1, V, dtype=np.float64)           # ids 1..V-1; id 0 is the CLS marker
    cdf = np.cumsum(ranks ** (-a))
    cdf /= cdf[-1]
    u = rng.uniform(stream, n_seq * S)
    ids = np.minimum(np.searchsorted(cdf, u, side="right") + 1, V - 1).astype(np.int32).reshape(n_seq, S)
    ids[:, 0] = 0
    return ids


# Auxiliary-task reweighting (Sec. 4.3 runs it on RoBERTa-base): the encoder of workload 4 with RoBERTa's vocabulary
# (50265, rounded up to the next multiple of 64 as the masked-token head requires) and that workload's optimiser
# settings; 16 finetuning + 16 auxiliary sequences per base step, 16 meta sequences, 256 tokens each (the batch size and the
# maximum sequence length App. B gives for those runs).
AUX_TASK = dict(base=4, dims=(12, 768, 12, 3072, 256, 50304, 6), batch=16, meta_batch=16, n_pt=16)


def make_aux_workload(n_train=None, n_meta=None, **override):
    kw = dict(dims=AUX_TASK["dims"], batch=AUX_TASK["batch"], meta_batch=AUX_TASK["meta_batch"], mlm=True)
    kw.update(override)
    return make_workload(AUX_TASK["base"], n_train=n_train, n_meta=n_meta, **kw)


def make_aux_batch(wl, step, n_pt, lo=0.10, hi=0.20):
    """Masked-token batch `step` of the auxiliary task of an encoder workload: n_pt sequences of the token recipe
    (own stream), in each a seeded choice of between lo*S and hi*S positions (never position 0) whose ids are replaced
    by the mask id V-1 in the input and kept as targets.  Returns (ids [n_pt, S] int32, seq [n_mask] int32,
    pos [n_mask] int32, tgt [n_mask] int32) with (seq, pos) ascending."""
    L, d, heads, ffn, S, V, C = wl.dims
    rng = CounterRNG(wl.seed + 7919 * (step + 1))
    ids = _zipf_tokens(rng, S_TOK_AUX, n_pt, S, V)
    k = np.floor(S * (lo + (hi - lo) * rng.uniform(S_AUX_COUNT, n_pt))).astype(np.int64).clip(1, S - 1)
    seq, pos = [], []
    for i in range(n_pt):
        p = np.sort(1 + rng.permutation(S_AUX_PERM + i, S - 1)[:k[i]])
        seq.append(np.full(len(p), i)); pos.append(p)
    seq, pos = np.concatenate(seq).astype(np.int32), np.concatenate(pos).astype(np.int32)
    tgt = ids[seq, pos].astype(np.int32)
    ids[seq, pos] = V - 1
    return ids, seq, pos, tgt


def seq_lengths(seed, n, S, lo=0.15):
    """A length mix for n padded sequences of at most S tokens, as short texts give it: log-uniform between lo*S and
    2*S, cut at S, so that about a quarter of the sequences fill all S positions (truncated texts) and the rest spread
    down to a few tokens.  int32 [n], each in [1, S]."""
    u = CounterRNG(seed).uniform(S_LENGTHS, n)
    a, b = np.log(max(lo * S, 1.0)), np.log(2.0 * S)
    return np.clip(np.floor(np.exp(a + (b - a) * u)), 1, S).astype(np.int32)


def make_workload(cfg, n_train=None, n_meta=None, **override):
    """Build workload `cfg` (1..5).  n_train / n_meta may shrink the data set for quick tests
    (the first rows of the full recipe are NOT guaranteed identical when shrunk); `override`
    replaces other fields (dims, batch, ...) to get a small model on the same data recipe."""
    kw = dict(WORKLOADS[cfg])
    kw.update(override)
    if n_train is not None:
        kw["n_train"] = n_train
    if n_meta is not None:
        kw["n_meta"] = n_meta
    wl = Workload(cfg=cfg, **kw)
    rng = CounterRNG(wl.seed)
    C = wl.n_classes
    if cfg == 1:
        F = wl.dims[0]
        T = rng.normal(S_TEACHER, F * C).reshape(F, C)
        X = rng.normal(S_X, wl.n_train * F).reshape(wl.n_train, F).astype(np.float32)
        Xm = rng.normal(S_XMETA, wl.n_meta * F).reshape(wl.n_meta, F).astype(np.float32)
        y = np.argmax(X.astype(np.float64) @ T, axis=1).astype(np.int32)
        ym = np.argmax(Xm.astype(np.float64) @ T, axis=1).astype(np.int32)
    elif cfg == 2:
        F = wl.dims[0]
        means = 2.0 * rng.normal(S_MEANS, C * F).reshape(C, F)
        y = rng.integers(S_CLASS, wl.n_train, C).astype(np.int32)
        ym = rng.integers(S_CLASS_META, wl.n_meta, C).astype(np.int32)
        X = (means[y] + rng.normal(S_X, wl.n_train * F).reshape(wl.n_train, F)).astype(np.float32)
        Xm = (means[ym] + rng.normal(S_XMETA, wl.n_meta * F).reshape(wl.n_meta, F)).astype(np.float32)
    else:
        L, d, heads, ffn, S, V, C = wl.dims
        T = rng.normal(S_TEACHER, V * C).reshape(V, C)
        X = _zipf_tokens(rng, S_TOK, wl.n_train, S, V)
        Xm = _zipf_tokens(rng, S_TOK_META, wl.n_meta, S, V)
        y = np.argmax(T[X].sum(axis=1), axis=1).astype(np.int32)
        ym = np.argmax(T[Xm].sum(axis=1), axis=1).astype(np.int32)
    y_noisy, flipped = flip_labels(rng, y, C, wl.noise)
    wl.x_train, wl.y_train, wl.y_train_clean, wl.flipped = X, y_noisy.astype(np.int32), y, flipped
    wl.x_meta, wl.y_meta = Xm, ym
    return wl
