"""Seeded synthetic kernel traces of DNN training steps.

A trace is what the offline profiling stage of the paper hands to the planner
(Section 4.2): the ordered kernel list with one profiled duration per kernel,
the tensors each kernel touches, every tensor's byte size, and which tensors
are global (weights and optimizer state, alive across iterations) as opposed
to intermediate (activations, gradients, workspaces).

This module only *describes workloads*.  It contains none of the planner's
arithmetic: no use lists, no lifetimes, no pressure, no capacity.  A workload
carries the capacity as a *fraction of the peak footprint*; whoever runs the
vitality analysis turns that into bytes.  Both the CPU oracle's tests and the
GPU path's tests/bench draw their inputs from here.

Randomness is a counter-based generator written below (SplitMix64 finaliser
over seed/stream/index), so any element of any stream can be computed on its
own and the arrays do not depend on a library RNG.

The five workloads stand in for the profiled traces of Table 1 (BERT, ViT,
Inceptionv3, ResNet152, SENet154: 740-2318 kernels each), which are not
available here; they follow Section 3's characterisation: tensors are used
about twice (forward and backward), sizes span KB to GB, single-use
workspaces exist (Figure 6), and weights are re-used by the next iteration.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

_U64 = np.uint64
_MASK = (1 << 64) - 1


# ----------------------------------------------------------------------------
# counter-based random numbers
# ----------------------------------------------------------------------------
def _mix(x: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        x = (x ^ (x >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> _U64(27))) * _U64(0x94D049BB133111EB)
        x = x ^ (x >> _U64(31))
    return x


def rand_u64(seed: int, stream: int, idx) -> np.ndarray:
    """Random 64-bit words: element i of stream `stream` under `seed`."""
    idx = np.asarray(idx, dtype=np.uint64)
    base = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03) & _MASK
    with np.errstate(over="ignore"):
        x = _U64(base) + (idx + _U64(1)) * _U64(0x9E3779B97F4A7C15)
    return _mix(_mix(x) ^ _U64(base))


def rand_unit(seed: int, stream: int, idx) -> np.ndarray:
    """Doubles in the open interval (0, 1)."""
    r = rand_u64(seed, stream, idx)
    return ((r >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def rand_int(seed: int, stream: int, idx, lo: int, hi: int) -> np.ndarray:
    """Integers in [lo, hi] (inclusive)."""
    r = rand_u64(seed, stream, idx)
    return (r % _U64(hi - lo + 1)).astype(np.int64) + lo


def rand_lognormal_ns(seed: int, stream: int, n: int, median_ns: float, sigma: float) -> np.ndarray:
    """n kernel durations, log-normal around `median_ns`, rounded to >= 1 ns."""
    i = np.arange(n, dtype=np.uint64)
    u1 = rand_unit(seed, stream, i)
    u2 = rand_unit(seed, stream + 1, i)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)   # Box-Muller
    d = np.rint(np.exp(math.log(median_ns) + sigma * z))
    return np.maximum(d, 1.0).astype(np.uint64)


# ----------------------------------------------------------------------------
# containers
# ----------------------------------------------------------------------------
@dataclass
class Trace:
    """One training step as the planner sees it (all arrays are host numpy)."""
    name: str
    dur_ns: np.ndarray        # [K] uint64, > 0
    size_bytes: np.ndarray    # [N] uint64, > 0
    is_global: np.ndarray     # [N] uint8
    use_kernel: np.ndarray    # [P] uint32  (COO, any order, duplicates legal)
    use_tensor: np.ndarray    # [P] uint32

    @property
    def K(self) -> int:
        return int(self.dur_ns.shape[0])

    @property
    def N(self) -> int:
        return int(self.size_bytes.shape[0])

    @property
    def P(self) -> int:
        return int(self.use_kernel.shape[0])


@dataclass
class Workload:
    """A trace plus the machine it is planned for.

    Bandwidths are bytes per microsecond (6 GB/s = 6000), index 0 = flash
    (SSD), index 1 = host memory.  Capacities are fractions of the trace's
    peak footprint, to be resolved by the caller's own vitality analysis.
    """
    trace: Trace
    cap_frac: float
    host_cap_frac: float = 0.25
    bw_out_Bpus: tuple = (6000, 25000)
    bw_in_Bpus: tuple = (6000, 25000)
    meta: dict = field(default_factory=dict)


def resolve_caps(w: Workload, peak_bytes: int) -> tuple:
    """(gpu_cap, host_cap) in bytes from the workload's fractions (floor)."""
    num, den = _frac(w.cap_frac)
    hnum, hden = _frac(w.host_cap_frac)
    return (peak_bytes * num) // den, (peak_bytes * hnum) // hden


def _frac(f: float) -> tuple:
    den = 10000
    return int(round(f * den)), den


# ----------------------------------------------------------------------------
# a small graph builder: forward ops are recorded, backward ops are derived
# ----------------------------------------------------------------------------
class _Graph:
    """Records kernels of a forward pass and derives backward + optimizer.

    Not an autograd: it only reproduces the *access pattern* of one, which is
    what the planner consumes (who touches which tensor, in which order).
    """

    def __init__(self, tmp_seed: int = 0, fwd_tmps: int = 0, bwd_tmps: int = 0, opt_tmps: int = 0,
                 tmp_log2: tuple = (16, 23)):
        # Single-use temporaries (the pattern of Figure 6's tensor2914: allocated for one kernel, never
        # used again): every forward / backward / optimizer kernel gets this many, sized log-uniformly
        # between 2^tmp_log2[0] and 2^tmp_log2[1] bytes from a counter-based stream of their own.
        self.tmp_seed, self.tmp_log2 = tmp_seed, tmp_log2
        self.tmps = dict(fwd=fwd_tmps, bwd=bwd_tmps, opt=opt_tmps)
        self.phase = "fwd"
        self.n_tmp = 0
        self.sizes: list = []
        self.glob: list = []
        self.kernels: list = []          # list of list of tensor ids
        self.fwd: list = []              # recorded forward ops for backward
        self.grad: dict = {}             # tensor id -> gradient tensor id
        self.weights: list = []          # weight ids in creation order

    # tensors -------------------------------------------------------------
    def tensor(self, nbytes: int, is_global: bool = False) -> int:
        assert nbytes > 0
        self.sizes.append(int(nbytes))
        self.glob.append(1 if is_global else 0)
        return len(self.sizes) - 1

    def weight(self, nbytes: int) -> int:
        w = self.tensor(nbytes, True)
        self.weights.append(w)
        return w

    def grad_of(self, t: int) -> int:
        if t not in self.grad:
            self.grad[t] = self.tensor(self.sizes[t], False)
        return self.grad[t]

    # kernels -------------------------------------------------------------
    def kernel(self, uses) -> int:
        uses = [int(u) for u in uses]
        for _ in range(self.tmps[self.phase]):
            lo, hi = self.tmp_log2
            e = lo + (hi - lo) * float(rand_unit(self.tmp_seed, 7, np.array([self.n_tmp]))[0])
            uses.append(self.tensor(max(4096, int(2.0 ** e)) & ~255))
            self.n_tmp += 1
        self.kernels.append(uses)
        return len(self.kernels) - 1

    def op(self, ins, ws, outs, saved=None, ws_bytes: int = 0, extra=()):
        """Forward kernel reading activations `ins` and weights `ws`,
        writing `outs`.  `saved` = tensors its backward needs (default: ins).
        `ws_bytes` > 0 adds a single-use workspace tensor (Figure 6's
        tensor2914 pattern) to the forward and to each backward kernel."""
        uses = list(ins) + list(ws) + list(outs) + list(extra)
        if ws_bytes:
            uses.append(self.tensor(ws_bytes))
        self.kernel(uses)
        self.fwd.append(dict(ins=list(ins), ws=list(ws), outs=list(outs),
                             saved=list(ins) if saved is None else list(saved),
                             ws_bytes=ws_bytes))

    def backward(self, split_weight_grads: bool = True):
        """Emit backward kernels in reverse order of the recorded forward."""
        self.phase = "bwd"
        for rec in reversed(self.fwd):
            douts = [self.grad_of(o) for o in rec["outs"]]
            if rec["ins"]:
                dins = [self.grad_of(i) for i in rec["ins"]]
                uses = douts + rec["saved"] + rec["ws"] + dins
                if rec["ws_bytes"]:
                    uses.append(self.tensor(rec["ws_bytes"]))
                self.kernel(uses)
            if rec["ws"]:
                groups = [[w] for w in rec["ws"]] if split_weight_grads else [rec["ws"]]
                for g in groups:
                    uses = douts + rec["ins"] + [self.grad_of(w) for w in g]
                    if rec["ws_bytes"]:
                        uses.append(self.tensor(rec["ws_bytes"]))
                    self.kernel(uses)
        self.fwd = []

    def optimizer(self, n_state: int, n_kernels: int, half_copy: bool = False, fp32_grad: bool = False,
                  pre_kernels: int = 0):
        """Per weight: `n_state` fp32 state tensors (momentum / Adam moments),
        an update split over `n_kernels` elementwise kernels, optionally a
        half-precision working copy refreshed by a cast kernel.  `fp32_grad`:
        the half-precision gradient is first accumulated into an fp32 buffer
        that lives across iterations (one more kernel and tensor per weight).
        `pre_kernels`: elementwise kernels on the gradient alone before the
        update (unscale / average over replicas / clip)."""
        self.phase = "opt"
        for w in self.weights:
            if w not in self.grad:
                continue
            g = self.grad[w]
            for _ in range(pre_kernels):
                self.kernel([g])
            if fp32_grad:
                acc = self.tensor(self.sizes[w] * 2, True)
                self.kernel([g, acc])
                g = acc
            states = [self.tensor(self.sizes[w], True) for _ in range(n_state)]
            for j in range(n_kernels):
                s = states[j % n_state] if n_state else None
                uses = [w, g] + ([s] if s is not None else [])
                if j == n_kernels - 1:
                    uses = [w, g] + states
                self.kernel(uses)
            if half_copy:
                h = self.tensor(max(1, self.sizes[w] // 2), True)
                self.kernel([w, h])

    # output --------------------------------------------------------------
    def finish(self, name: str, dur_ns: np.ndarray) -> Trace:
        K = len(self.kernels)
        assert dur_ns.shape[0] == K
        uk = np.fromiter((k for k, us in enumerate(self.kernels) for _ in us), dtype=np.uint32)
        ut = np.fromiter((u for us in self.kernels for u in us), dtype=np.uint32)
        return Trace(name, dur_ns.astype(np.uint64),
                     np.asarray(self.sizes, dtype=np.uint64),
                     np.asarray(self.glob, dtype=np.uint8), uk, ut)


# ----------------------------------------------------------------------------
# config 1: tiny 4-layer MLP, fp32, batch 64, hidden 256
# ----------------------------------------------------------------------------
def mlp_tiny(seed: int = 0x67100001) -> Workload:
    B, H, L = 64, 256, 4
    g = _Graph()
    act, wsz, bsz = B * H * 4, H * H * 4, H * 4
    A = [g.tensor(act)]
    W = [g.weight(wsz) for _ in range(L)]
    b = [g.weight(bsz) for _ in range(L)]
    Z = []
    for l in range(L):                                   # forward: GEMM, ReLU
        Z.append(g.tensor(act))
        g.kernel([A[l], W[l], b[l], Z[l]])
        A.append(g.tensor(act))
        g.kernel([Z[l], A[l + 1]])
    dA = {L: g.tensor(act)}
    dW, db = {}, {}
    for l in reversed(range(L)):                         # backward: dReLU, dX, dW
        dZ = g.tensor(act)
        g.kernel([dA[l + 1], Z[l], dZ])
        dA[l] = g.tensor(act)
        g.kernel([dZ, W[l], dA[l]])
        dW[l], db[l] = g.tensor(wsz), g.tensor(bsz)
        g.kernel([dZ, A[l], dW[l], db[l]])
    for l in range(L):                                   # SGD
        g.kernel([W[l], dW[l], b[l], db[l]])
    K = len(g.kernels)
    dur = rand_int(seed, 1, np.arange(K), 5_000, 50_000).astype(np.uint64)
    return Workload(g.finish("mlp4", dur), cap_frac=0.60,
                    meta=dict(config=1, batch=B, hidden=H, layers=L))


# ----------------------------------------------------------------------------
# config 2: 12-layer transformer encoder, fp16 activations, fp32 master weights
# ----------------------------------------------------------------------------
def _linear(g: _Graph, x: int, d_in: int, d_out: int, rows: int, esz: int, wsz: int,
            ws_bytes: int = 0) -> int:
    """GEMM kernel then a separate bias-add kernel; returns the output id."""
    w = g.weight(d_in * d_out * wsz)
    b = g.weight(d_out * wsz)
    y = g.tensor(rows * d_out * esz)
    g.op([x], [w], [y], ws_bytes=ws_bytes)
    yb = g.tensor(rows * d_out * esz)
    g.op([y], [b], [yb], saved=[])
    return yb


def _norm(g: _Graph, x: int, d: int, rows: int, esz: int, wsz: int, affine_bias: bool = True) -> int:
    gam = g.weight(d * wsz)
    ws = [gam] + ([g.weight(d * wsz)] if affine_bias else [])
    y = g.tensor(rows * d * esz)
    stat = g.tensor(rows * 4 * (2 if affine_bias else 1))        # saved mean / rstd
    g.op([x], ws, [y], saved=[x, stat], extra=[stat])
    return y


def encoder12(seed: int = 0x67100002) -> Workload:
    Bt, S, H, NH, L, FF, V = 32, 512, 768, 12, 12, 3072, 30522
    esz, wsz = 2, 4
    rows = Bt * S
    g = _Graph(tmp_seed=seed, fwd_tmps=1, bwd_tmps=2)             # every kernel with scratch of its own, single use
    ids = g.tensor(rows * 8)
    emb = g.weight(V * H * wsz)
    pos = g.weight(S * H * wsz)
    x = g.tensor(rows * H * esz)
    g.op([], [emb, pos], [x], extra=[ids])
    x = _norm(g, x, H, rows, esz, wsz)
    mask = g.tensor(Bt * S * esz)
    for _ in range(L):
        h = _norm(g, x, H, rows, esz, wsz)
        qkv = _linear(g, h, H, 3 * H, rows, esz, wsz, ws_bytes=4 << 20)
        q, k, v = (g.tensor(rows * H * esz) for _ in range(3))
        for o in (q, k, v):
            g.op([qkv], [], [o], saved=[])
        sc = g.tensor(Bt * NH * S * S * esz)
        g.op([q, k], [], [sc])
        sc2 = g.tensor(Bt * NH * S * S * esz)
        g.op([sc], [], [sc2], saved=[], extra=[mask])
        pr = g.tensor(Bt * NH * S * S * esz)
        g.op([sc2], [], [pr], saved=[pr])
        dm = g.tensor(Bt * NH * S * S)                           # dropout mask, 1 byte
        prd = g.tensor(Bt * NH * S * S * esz)
        g.op([pr], [], [prd], saved=[dm], extra=[dm])
        ctx = g.tensor(rows * H * esz)
        g.op([prd, v], [], [ctx])
        ctxm = g.tensor(rows * H * esz)
        g.op([ctx], [], [ctxm], saved=[])
        o = _linear(g, ctxm, H, H, rows, esz, wsz, ws_bytes=4 << 20)
        dm2 = g.tensor(rows * H)
        od = g.tensor(rows * H * esz)
        g.op([o], [], [od], saved=[dm2], extra=[dm2])
        x1 = g.tensor(rows * H * esz)
        g.op([od, x], [], [x1], saved=[])
        h2 = _norm(g, x1, H, rows, esz, wsz)
        f1 = _linear(g, h2, H, FF, rows, esz, wsz, ws_bytes=4 << 20)
        ge = g.tensor(rows * FF * esz)
        g.op([f1], [], [ge])
        f2 = _linear(g, ge, FF, H, rows, esz, wsz, ws_bytes=4 << 20)
        dm3 = g.tensor(rows * H)
        fd = g.tensor(rows * H * esz)
        g.op([f2], [], [fd], saved=[dm3], extra=[dm3])
        x2 = g.tensor(rows * H * esz)
        g.op([fd, x1], [], [x2], saved=[])
        x = x2
    pooled = g.tensor(Bt * H * esz)
    g.op([x], [], [pooled])
    logits = _linear(g, pooled, H, 2, Bt, esz, wsz)
    labels = g.tensor(Bt * 8)
    loss = g.tensor(4)
    g.op([logits], [], [loss], saved=[logits], extra=[labels])
    g.backward(split_weight_grads=True)
    g.optimizer(n_state=2, n_kernels=2, half_copy=True, fp32_grad=True)   # fp32 gradient accumulation, AdamW, cast
    K = len(g.kernels)
    dur = rand_lognormal_ns(seed, 1, K, 80_000.0, 1.0)
    return Workload(g.finish("encoder12", dur), cap_frac=0.50,
                    meta=dict(config=2, batch=Bt, seq=S, hidden=H, layers=L))


# ----------------------------------------------------------------------------
# config 3: 152-layer residual CNN (bottleneck blocks), fp32, batch 256
# ----------------------------------------------------------------------------
def _conv_bn(g: _Graph, x: int, n: int, cin: int, cout: int, hw: int, ksz: int, relu: bool) -> int:
    esz = 4
    w = g.weight(cin * cout * ksz * ksz * esz)
    out_b = n * cout * hw * hw * esz
    col = g.tensor(max(4096, min(out_b, 256 << 20)))             # transform / im2col scratch
    g.op([x], [], [col], saved=[])
    wt = g.tensor(cin * cout * ksz * ksz * esz)                  # filter in the layout the convolution kernel wants
    g.op([], [w], [wt])
    yt = g.tensor(out_b)
    g.op([col, wt], [], [yt], saved=[x, wt], ws_bytes=64 << 20)
    y = g.tensor(out_b)                                           # output back in the activation layout
    g.op([yt], [], [y], saved=[])
    gam, bet = g.weight(cout * esz), g.weight(cout * esz)
    rm, rv = g.tensor(cout * esz, True), g.tensor(cout * esz, True)
    mean, var = g.tensor(cout * esz), g.tensor(cout * esz)
    g.op([y], [], [mean, var], saved=[])                           # batch statistics
    g.kernel([mean, var, rm, rv])                                  # running statistics (no backward)
    yn = g.tensor(out_b)                                          # normalised, kept for the backward of the affine part
    g.op([y], [], [yn], saved=[y, mean, var], extra=[mean, var])
    z = g.tensor(out_b)
    g.op([yn], [gam, bet], [z], saved=[yn])
    if relu:
        r = g.tensor(out_b)
        g.op([z], [], [r], saved=[r])
        return r
    return z


def resnet152(seed: int = 0x67100003) -> Workload:
    n, esz = 256, 4
    g = _Graph(tmp_seed=seed, fwd_tmps=1, bwd_tmps=2, opt_tmps=2)
    img = g.tensor(n * 3 * 224 * 224 * esz)
    x = _conv_bn(g, img, n, 3, 64, 112, 7, True)
    p = g.tensor(n * 64 * 56 * 56 * esz)
    g.op([x], [], [p], saved=[x, p])
    x, cin, hw = p, 64, 56
    for stage, (blocks, mid) in enumerate(zip((3, 8, 36, 3), (64, 128, 256, 512))):
        cout = mid * 4
        for bi in range(blocks):
            if bi == 0 and stage > 0:
                hw //= 2
            y = _conv_bn(g, x, n, cin, mid, hw, 1, True)
            y = _conv_bn(g, y, n, mid, mid, hw, 3, True)
            y = _conv_bn(g, y, n, mid, cout, hw, 1, False)
            sc = _conv_bn(g, x, n, cin, cout, hw, 1, False) if bi == 0 else x
            s = g.tensor(n * cout * hw * hw * esz)
            g.op([y, sc], [], [s], saved=[])
            r = g.tensor(n * cout * hw * hw * esz)
            g.op([s], [], [r], saved=[r])
            x, cin = r, cout
    pooled = g.tensor(n * cin * esz)
    g.op([x], [], [pooled], saved=[])
    fcw, fcb = g.weight(cin * 1000 * esz), g.weight(1000 * esz)
    logits = g.tensor(n * 1000 * esz)
    g.op([pooled], [fcw, fcb], [logits])
    labels = g.tensor(n * 8)
    loss = g.tensor(4)
    g.op([logits], [], [loss], saved=[logits], extra=[labels])
    g.backward(split_weight_grads=True)
    g.optimizer(n_state=1, n_kernels=4, pre_kernels=2)            # average over replicas, clip; decay, momentum, update, statistics
    K = len(g.kernels)
    dur = rand_lognormal_ns(seed, 1, K, 80_000.0, 1.0)
    return Workload(g.finish("resnet152", dur), cap_frac=0.40,
                    bw_out_Bpus=(12000, 25000), bw_in_Bpus=(12000, 25000),
                    meta=dict(config=3, batch=n))


# ----------------------------------------------------------------------------
# config 4: 48-layer transformer decoder, bf16, hidden 4096, no recompute
# ----------------------------------------------------------------------------
def decoder48(seed: int = 0x67100004) -> Workload:
    Bt, S, H, NH, L, FF, V = 16, 2048, 4096, 32, 48, 16384, 32000
    HG = 16                                   # attention runs per group of NH/HG heads
    esz, wsz = 2, 2
    rows = Bt * S
    g = _Graph(tmp_seed=seed, fwd_tmps=2, bwd_tmps=2, opt_tmps=2)
    ids = g.tensor(rows * 8)
    emb = g.weight(V * H * wsz)
    x = g.tensor(rows * H * esz)
    g.op([], [emb], [x], extra=[ids])
    rope = g.tensor(S * (H // NH) * 4, True)
    gsz = rows * (H // HG) * esz              # one head group's slice of q / k / v / ctx
    ssz = Bt * (NH // HG) * S * S * esz       # one head group's score matrix
    for _ in range(L):
        h = _norm(g, x, H, rows, esz, wsz, affine_bias=False)
        wq, wk, wv = (g.weight(H * H * wsz) for _ in range(3))
        q, k, v = (g.tensor(rows * H * esz) for _ in range(3))
        for w, o in ((wq, q), (wk, k), (wv, v)):
            g.op([h], [w], [o], ws_bytes=32 << 20)
        qr, kr = g.tensor(rows * H * esz), g.tensor(rows * H * esz)
        g.op([q], [], [qr], saved=[], extra=[rope])
        g.op([k], [], [kr], saved=[], extra=[rope])
        ctx_parts = []
        for _hg in range(HG):
            qg, kg, vg = (g.tensor(gsz) for _ in range(3))
            g.op([qr], [], [qg], saved=[])
            g.op([kr], [], [kg], saved=[])
            g.op([v], [], [vg], saved=[])
            sc = g.tensor(ssz)
            g.op([qg, kg], [], [sc])
            pr = g.tensor(ssz)
            lse = g.tensor(Bt * (NH // HG) * S * 4)
            g.op([sc], [], [pr], saved=[pr, lse], extra=[lse])
            cg = g.tensor(gsz)
            g.op([pr, vg], [], [cg])
            ctx_parts.append(cg)
        ctx = g.tensor(rows * H * esz)
        g.op(ctx_parts, [], [ctx], saved=[])
        wo = g.weight(H * H * wsz)
        o = g.tensor(rows * H * esz)
        g.op([ctx], [wo], [o], ws_bytes=32 << 20)
        x1 = g.tensor(rows * H * esz)
        g.op([o, x], [], [x1], saved=[])
        h2 = _norm(g, x1, H, rows, esz, wsz, affine_bias=False)
        wg, wu, wd = g.weight(H * FF * wsz), g.weight(H * FF * wsz), g.weight(FF * H * wsz)
        gt, up = g.tensor(rows * FF * esz), g.tensor(rows * FF * esz)
        g.op([h2], [wg], [gt], ws_bytes=32 << 20)
        g.op([h2], [wu], [up], ws_bytes=32 << 20)
        act = g.tensor(rows * FF * esz)
        g.op([gt, up], [], [act])
        dn = g.tensor(rows * H * esz)
        g.op([act], [wd], [dn], ws_bytes=32 << 20)
        x2 = g.tensor(rows * H * esz)
        g.op([dn, x1], [], [x2], saved=[])
        x = x2
    hN = _norm(g, x, H, rows, esz, wsz, affine_bias=False)
    lm = g.weight(H * V * wsz)
    logits = g.tensor(rows * V * esz)         # 2.1 GB: the largest tensor
    g.op([hN], [lm], [logits], ws_bytes=32 << 20)
    labels = g.tensor(rows * 8)
    loss = g.tensor(4)
    g.op([logits], [], [loss], saved=[logits], extra=[labels])
    g.backward(split_weight_grads=True)
    g.optimizer(n_state=3, n_kernels=3)       # fp32 master + two Adam moments
    K = len(g.kernels)
    dur = rand_lognormal_ns(seed, 1, K, 200_000.0, 1.2)
    return Workload(g.finish("decoder48", dur), cap_frac=0.30,
                    meta=dict(config=4, batch=Bt, seq=S, hidden=H, layers=L))


# ----------------------------------------------------------------------------
# config 5: stress trace, parametrised so that scaled-down copies exist
# ----------------------------------------------------------------------------
def stress(K: int = 100_000, N: int = 1_000_000, seed: int = 0x67100005,
           cap_frac: float = 0.25, median_ns: float = 80_000.0, sigma: float = 1.0,
           min_log2: int = 12, max_log2: int = 29) -> Workload:
    """Forward/backward-mirrored lifetimes with Zipf-distributed extra uses.

    Tensor classes: 2 % global, 78 % mirrored (first use i in the first half,
    last use K-1-i), 20 % backward-local (born in the second half, dead 1..16
    kernels later).  Global tensors are touched at a forward kernel i and at
    its mirror K-1-i like weights.  Each kernel additionally touches 2..8
    tensors drawn with P(rank r) ~ r^-1.1 over the tensors alive at it, ranked
    by recency of birth; about 1 % of those draws are emitted twice (the same
    tensor passed twice to one kernel, as in Figure 6's ReLU).  Sizes are
    log-uniform in [2^min_log2, 2^max_log2] bytes.
    """
    assert K >= 8 and N >= 8
    half = K // 2
    t = np.arange(N, dtype=np.uint64)
    cls = rand_unit(seed, 10, t)
    is_glob = cls < 0.02
    is_loc = cls >= 0.80
    first = rand_int(seed, 11, t, 0, half - 1)
    last = (K - 1) - first
    lb = rand_int(seed, 12, t, half, K - 1)
    le = np.minimum(K - 1, lb + rand_int(seed, 13, t, 1, 16))
    first = np.where(is_loc, lb, first)
    last = np.where(is_loc, le, last)
    size = np.floor(np.exp2(min_log2 + (max_log2 - min_log2) * rand_unit(seed, 14, t)))
    size = np.clip(size, 1 << min_log2, 1 << max_log2).astype(np.uint64)

    uk = [first.astype(np.uint32), last.astype(np.uint32)]
    ut = [t.astype(np.uint32), t.astype(np.uint32)]

    # extra uses: ranked list = forward-born tensors sorted by first use
    fw = np.flatnonzero(~is_loc)
    order = fw[np.argsort(first[fw], kind="stable")]
    fsorted = first[order]
    k = np.arange(K, dtype=np.int64)
    n_alive = np.searchsorted(fsorted, np.minimum(k, K - 1 - k), side="right")
    m = rand_int(seed, 20, k, 2, 8)
    rep = np.repeat(k, m)                                        # kernel of each draw
    j = np.arange(rep.shape[0], dtype=np.uint64)
    na = n_alive[rep]
    ok = na > 0
    rep, j, na = rep[ok], j[ok], na[ok].astype(np.float64)
    s = 1.1
    u = rand_unit(seed, 21, j)
    r = np.floor((u * (np.power(na + 1.0, 1.0 - s) - 1.0) + 1.0) ** (1.0 / (1.0 - s)))
    r = np.clip(r, 1.0, na).astype(np.int64)
    pick = order[na.astype(np.int64) - r]
    uk.append(rep.astype(np.uint32))
    ut.append(pick.astype(np.uint32))
    dup = rand_unit(seed, 22, j) < 0.01
    uk.append(rep[dup].astype(np.uint32))
    ut.append(pick[dup].astype(np.uint32))

    # backward-local tensors: 0..2 extra touches inside their short lifetime
    loc = np.flatnonzero(is_loc)
    for rnd in range(2):
        take = rand_unit(seed, 30 + rnd, loc.astype(np.uint64)) < 0.5
        tl = loc[take]
        span = (last[tl] - first[tl] + 1).astype(np.uint64)
        kk = first[tl] + (rand_u64(seed, 32 + rnd, tl.astype(np.uint64)) % span).astype(np.int64)
        uk.append(kk.astype(np.uint32))
        ut.append(tl.astype(np.uint32))

    use_kernel = np.concatenate(uk)
    use_tensor = np.concatenate(ut)
    perm = np.argsort(rand_u64(seed, 40, np.arange(use_kernel.shape[0])), kind="stable")
    dur = rand_lognormal_ns(seed, 1, K, median_ns, sigma)
    tr = Trace(f"stress_K{K}_N{N}", dur, size, is_glob.astype(np.uint8),
               use_kernel[perm], use_tensor[perm])
    return Workload(tr, cap_frac=cap_frac, meta=dict(config=5, K=K, N=N))


def noisy_durations(tr: Trace, percent: float, seed: int) -> np.ndarray:
    """The trace's kernel durations with a profiling error of up to +-`percent` % on each
    (uniform, independent per kernel), rounded to >= 1 ns: the input of a re-planning
    study under kernel-time noise."""
    i = np.arange(tr.K, dtype=np.uint64)
    f = 1.0 + (2.0 * rand_unit(seed, 77, i) - 1.0) * (percent / 100.0)
    return np.maximum(np.rint(tr.dur_ns.astype(np.float64) * f), 1.0).astype(np.uint64)


def with_durations(tr: Trace, dur_ns: np.ndarray) -> Trace:
    """The same step with other kernel durations."""
    return Trace(tr.name + "_dur", np.ascontiguousarray(dur_ns, np.uint64), tr.size_bytes, tr.is_global,
                 tr.use_kernel, tr.use_tensor)


def config(i: int) -> Workload:
    """The five workloads of the benchmark, 1-based."""
    return {1: mlp_tiny, 2: encoder12, 3: resnet152, 4: decoder48, 5: stress}[i]()


def random_small(seed: int, K: int = 12, N: int = 8, max_uses: int = 4,
                 frac_global: float = 0.3) -> Workload:
    """Small random traces for property and brute-force tests.  Includes
    unused tensors, duplicate pairs and single-use tensors on purpose."""
    t = np.arange(N, dtype=np.uint64)
    glob = (rand_unit(seed, 1, t) < frac_global).astype(np.uint8)
    size = rand_int(seed, 2, t, 1, 64).astype(np.uint64) * np.uint64(1000)
    nuse = rand_int(seed, 3, t, 0, max_uses)
    rep = np.repeat(np.arange(N), nuse)
    j = np.arange(rep.shape[0], dtype=np.uint64)
    uk = rand_int(seed, 4, j, 0, K - 1)
    dur = rand_int(seed, 5, np.arange(K), 1, 20).astype(np.uint64) * np.uint64(1000)
    dup = rand_unit(seed, 6, j) < 0.1
    use_kernel = np.concatenate([uk, uk[dup]]).astype(np.uint32)
    use_tensor = np.concatenate([rep, rep[dup]]).astype(np.uint32)
    if use_kernel.shape[0] == 0:
        use_kernel = np.zeros(1, np.uint32)
        use_tensor = np.zeros(1, np.uint32)
    cap = 0.3 + 0.69 * float(rand_unit(seed, 7, [0])[0])
    bw_s = int(rand_int(seed, 8, [0], 300, 6000)[0])
    bw_h = int(rand_int(seed, 8, [1], 2000, 40000)[0])
    tr = Trace(f"rand{seed}", dur, size, glob, use_kernel, use_tensor)
    return Workload(tr, cap_frac=cap, host_cap_frac=float(rand_unit(seed, 9, [0])[0]) * 0.5,
                    bw_out_Bpus=(bw_s, bw_h), bw_in_Bpus=(bw_s + int(rand_int(seed, 8, [2], 0, 300)[0]), bw_h))
