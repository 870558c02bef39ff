"""Operator traces shaped like one training iteration (forward, backward,
optimizer) of the networks the benchmark configurations name.

Only shapes matter here: each function appends operators to a ``Trace`` and
tensor sizes are ``4 * prod(shape)`` bytes (fp32).  The layer shapes are the
standard published ones (MLP 784-512-256-10; ResNet-50 stages [3,4,6,3] with
bottleneck widths 64..512; VGG-16 configuration D; BERT-base 12 x 768 x 12
heads x 3072).  Nothing is trained or executed.

Every iteration function takes the state tensors it continues from
(parameters, Adam first and second moments) and returns their successors, so
iterations can be concatenated: an optimizer-phase tensor of one iteration is
read in the forward and backward phases of the next one (the paper's
across-iteration case, section IV-C).
"""
from __future__ import annotations

from math import prod
from typing import Dict, List, Sequence, Tuple

from .tas import Trace

F32 = 4


def nbytes(*shape: int) -> int:
    return F32 * prod(shape)


class Params:
    """Ordered parameter set with Adam state: name -> tensor id."""

    def __init__(self) -> None:
        self.names: List[str] = []
        self.shape: Dict[str, Tuple[int, ...]] = {}
        self.p: Dict[str, int] = {}
        self.m: Dict[str, int] = {}
        self.v: Dict[str, int] = {}


def placeholder(tr: Trace, shapes: Sequence[Tuple[str, Tuple[int, ...]]], tag: str = "") -> Params:
    """One placeholder operator that generates parameters and their Adam moments
    (the tensors resident when the first iteration begins)."""
    ps = Params()
    outs = []
    for name, shp in shapes:
        ps.names.append(name)
        ps.shape[name] = shp
        outs += [(f"{tag}{name}", nbytes(*shp)), (f"{tag}{name}.m", nbytes(*shp)), (f"{tag}{name}.v", nbytes(*shp))]
    ids = tr.op(outs=outs)
    for k, name in enumerate(ps.names):
        ps.p[name], ps.m[name], ps.v[name] = ids[3 * k], ids[3 * k + 1], ids[3 * k + 2]
    return ps


def adam(tr: Trace, ps: Params, grads: Dict[str, int], fine: bool, it: int, extra_reads: Sequence[int] = ()) -> Params:
    """Adam update of every parameter, in reverse order of creation (the order
    gradients become available).  ``fine`` spells out the temporaries of the
    textbook update (decayed gradient, bias-corrected moments, denominator,
    step) as tensors of their own.  Otherwise there are two operators per
    parameter, a fused in-place moment update and an in-place parameter update,
    software-pipelined by one parameter so that an in-place output is never
    read by the operator right after the one that wrote it."""
    new = Params()
    new.names, new.shape = ps.names, ps.shape
    order = list(reversed(ps.names))
    if not fine:
        def moments(name: str) -> None:
            b = nbytes(*ps.shape[name])
            new.m[name], new.v[name] = tr.op(reads=[ps.m[name], ps.v[name], grads[name], *extra_reads],
                                             inplace=[(f"i{it}.{name}.m", b), (f"i{it}.{name}.v", b)])

        def update(name: str) -> None:
            (new.p[name],) = tr.op(reads=[ps.p[name], new.m[name], new.v[name]],
                                   inplace=[(f"i{it}.{name}.new", nbytes(*ps.shape[name]))])

        moments(order[0])
        for prev, name in zip(order, order[1:]):
            moments(name)
            update(prev)
        update(order[-1])
        return new
    for name in order:
        b = nbytes(*ps.shape[name])
        g, p, m, v = grads[name], ps.p[name], ps.m[name], ps.v[name]
        t = f"i{it}.{name}"
        (g2,) = tr.op(reads=[g, p, *extra_reads], outs=[(f"{t}.gdecay", b)])
        (m2,) = tr.op(reads=[m, g2], inplace=[(f"{t}.m", b)])
        (v2,) = tr.op(reads=[v, g2], inplace=[(f"{t}.v", b)])
        (mh,) = tr.op(reads=[m2], outs=[(f"{t}.mhat", b)])
        (vh,) = tr.op(reads=[v2], outs=[(f"{t}.vhat", b)])
        (dn,) = tr.op(reads=[vh], outs=[(f"{t}.denom", b)])
        (up,) = tr.op(reads=[mh, dn], outs=[(f"{t}.step", b)])
        (p2,) = tr.op(reads=[p, up], inplace=[(f"{t}.new", b)])
        new.p[name], new.m[name], new.v[name] = p2, m2, v2
    return new


def finish(tr: Trace, ps: Params) -> None:
    """End of the trace: a synchronisation slot, then one operator that reads the
    final parameters and moments (they stay resident for the next iteration; the
    paper lists the parameters among the tensors in GPU memory when an iteration
    begins, section IV-B situation 1)."""
    tr.op()
    tr.op(reads=[t for name in ps.names for t in (ps.p[name], ps.m[name], ps.v[name])])


# --------------------------------------------------------------------------- MLP

MLP_DIMS = (784, 512, 256, 10)


def mlp_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    out = []
    for l in range(3):
        out += [(f"W{l + 1}", (MLP_DIMS[l], MLP_DIMS[l + 1])), (f"b{l + 1}", (MLP_DIMS[l + 1],))]
    return out


def mlp_iteration(tr: Trace, ps: Params, batch: int, it: int) -> Params:
    """3-layer MLP: per layer matmul, bias add, activation; softmax loss; the
    reverse sweep; gradient-norm clip; Adam.  With the placeholder this makes 60
    tensors for one iteration (20 state/input, 10 forward, 11 backward, 1 norm,
    18 optimizer outputs)."""
    t = f"i{it}"
    x, y = tr.op(outs=[(f"{t}.x", nbytes(batch, MLP_DIMS[0])), (f"{t}.y", nbytes(batch, MLP_DIMS[3]))])
    h = x
    saved = []
    for l in range(3):
        d = MLP_DIMS[l + 1]
        (z,) = tr.op(reads=[h, ps.p[f"W{l + 1}"]], outs=[(f"{t}.z{l + 1}", nbytes(batch, d))])
        (a,) = tr.op(reads=[z, ps.p[f"b{l + 1}"]], outs=[(f"{t}.a{l + 1}", nbytes(batch, d))])
        saved.append((h, a))
        if l < 2:
            (h,) = tr.op(reads=[a], outs=[(f"{t}.h{l + 1}", nbytes(batch, d))])
    probs, loss = tr.op(reads=[a, y], outs=[(f"{t}.probs", nbytes(batch, MLP_DIMS[3])), (f"{t}.loss", F32)])
    grads: Dict[str, int] = {}
    (da,) = tr.op(reads=[probs, y, loss], outs=[(f"{t}.da3", nbytes(batch, MLP_DIMS[3]))])
    for l in (2, 1, 0):
        h_in, a_l = saved[l]
        (grads[f"b{l + 1}"],) = tr.op(reads=[da], outs=[(f"{t}.db{l + 1}", nbytes(MLP_DIMS[l + 1]))])
        (grads[f"W{l + 1}"],) = tr.op(reads=[h_in, da], outs=[(f"{t}.dW{l + 1}", nbytes(MLP_DIMS[l], MLP_DIMS[l + 1]))])
        if l > 0:
            (dh,) = tr.op(reads=[da, ps.p[f"W{l + 1}"]], outs=[(f"{t}.dh{l}", nbytes(batch, MLP_DIMS[l]))])
            (da,) = tr.op(reads=[dh, saved[l - 1][1]], outs=[(f"{t}.da{l}", nbytes(batch, MLP_DIMS[l]))])
    (gn,) = tr.op(reads=list(grads.values()), outs=[(f"{t}.gnorm", F32)])
    return adam(tr, ps, grads, fine=False, it=it, extra_reads=[gn])


# ------------------------------------------------------------------- conv nets


class _ConvNet:
    """Shared bookkeeping for the convolutional traces: forward operators push
    what their backward operator needs on a tape that is replayed in reverse."""

    def __init__(self, tr: Trace, ps: Params, batch: int, it: int, workspace: bool) -> None:
        self.tr, self.ps, self.B, self.t, self.ws = tr, ps, batch, f"i{it}", workspace
        self.tape: List[tuple] = []
        self.grads: Dict[str, int] = {}
        self.n = 0

    def _nm(self, s: str) -> str:
        self.n += 1
        return f"{self.t}.{s}{self.n}"

    def conv(self, x: int, xs, name: str, cout: int, k: int, stride: int):
        c, h, w = xs
        ho, wo = (h + stride - 1) // stride, (w + stride - 1) // stride
        reads = [x, self.ps.p[name]]
        outs = [(self._nm("conv"), nbytes(self.B, cout, ho, wo))]
        if self.ws:
            outs.append((self._nm("ws"), min(nbytes(self.B, c * k * k, 64), 1 << 28)))
        ids = self.tr.op(reads=reads, outs=outs)
        self.tape.append(("conv", x, xs, name, k))
        return ids[0], (cout, ho, wo)

    def bias(self, x: int, xs, name: str):
        (y,) = self.tr.op(reads=[x, self.ps.p[name]], outs=[(self._nm("bias"), nbytes(self.B, *xs))])
        self.tape.append(("bias", name, xs))
        return y

    def bn(self, x: int, xs, name: str):
        c = xs[0]
        y, mean, istd = self.tr.op(reads=[x, self.ps.p[name + ".g"], self.ps.p[name + ".b"]],
                                   outs=[(self._nm("bn"), nbytes(self.B, *xs)), (self._nm("mean"), nbytes(c)),
                                         (self._nm("istd"), nbytes(c))])
        self.tr.op(reads=[mean, istd], outs=[(self._nm("rmean"), nbytes(c)), (self._nm("rvar"), nbytes(c))])
        self.tape.append(("bn", x, xs, name, mean, istd))
        return y

    def relu(self, x: int, xs):
        y, sign = self.tr.op(reads=[x], outs=[(self._nm("relu"), nbytes(self.B, *xs)),
                                              (self._nm("sign"), max(F32, nbytes(self.B, *xs) // 32))])
        self.tape.append(("relu", sign, xs))
        return y

    def pool(self, x: int, xs, stride: int):
        c, h, w = xs
        ys = (c, max(1, h // stride), max(1, w // stride))
        (y,) = self.tr.op(reads=[x], outs=[(self._nm("pool"), nbytes(self.B, *ys))])
        self.tape.append(("pool", x, y, xs))
        return y, ys

    def add(self, a: int, b: int, xs):
        (y,) = self.tr.op(reads=[a, b], outs=[(self._nm("add"), nbytes(self.B, *xs))])
        self.tape.append(("add", xs))
        return y

    def dropout(self, x: int, xs):
        y, mask = self.tr.op(reads=[x], outs=[(self._nm("drop"), nbytes(self.B, *xs)), (self._nm("mask"), nbytes(self.B, *xs) // 4)])
        self.tape.append(("drop", mask, xs))
        return y

    def fc(self, x: int, din: int, name: str, dout: int):
        (y,) = self.tr.op(reads=[x, self.ps.p[name + ".w"], self.ps.p[name + ".bias"]],
                          outs=[(self._nm("fc"), nbytes(self.B, dout))])
        self.tape.append(("fc", x, din, name, dout))
        return y

    def loss(self, logits: int, y: int, classes: int) -> int:
        probs, ls = self.tr.op(reads=[logits, y], outs=[(self._nm("probs"), nbytes(self.B, classes)), (self._nm("loss"), F32)])
        (d,) = self.tr.op(reads=[probs, y, ls], outs=[(self._nm("dlogits"), nbytes(self.B, classes))])
        return d


def _conv_backward(net: _ConvNet, dy: int, branch_grads: Dict[int, List[int]]) -> None:
    """Replay the tape in reverse.  ``branch_grads`` is unused for the purely
    sequential VGG; the residual nets handle their skip connections through the
    'fork'/'join' tape records below."""
    tr, ps, B = net.tr, net.ps, net.B
    stack: List[int] = []          # gradients parked for skip connections
    for rec in reversed(net.tape):
        kind = rec[0]
        if kind == "conv":
            _, x, xs, name, k = rec
            outs = [(net._nm("dw"), nbytes(*ps.shape[name]))]
            if net.ws:
                outs.append((net._nm("wsbf"), min(nbytes(B, xs[0] * k * k, 64), 1 << 28)))
            ids = tr.op(reads=[x, dy], outs=outs)
            net.grads[name] = ids[0]
            outs = [(net._nm("dx"), nbytes(B, *xs))]
            if net.ws:
                outs.append((net._nm("wsbd"), min(nbytes(B, xs[0] * k * k, 64), 1 << 28)))
            dy = tr.op(reads=[dy, ps.p[name]], outs=outs)[0]
        elif kind == "bias":
            _, name, xs = rec
            (net.grads[name],) = tr.op(reads=[dy], outs=[(net._nm("db"), nbytes(*ps.shape[name]))])
        elif kind == "bn":
            _, x, xs, name, mean, istd = rec
            dy, net.grads[name + ".g"], net.grads[name + ".b"] = tr.op(
                reads=[dy, x, mean, istd, ps.p[name + ".g"]],
                outs=[(net._nm("dbn"), nbytes(B, *xs)), (net._nm("dg"), nbytes(xs[0])), (net._nm("dbeta"), nbytes(xs[0]))])
        elif kind == "relu":
            _, sign, xs = rec
            (dy,) = tr.op(reads=[dy, sign], outs=[(net._nm("drelu"), nbytes(B, *xs))])
        elif kind == "pool":
            _, x, y, xs = rec
            (dy,) = tr.op(reads=[dy, x, y], outs=[(net._nm("dpool"), nbytes(B, *xs))])
        elif kind == "drop":
            _, mask, xs = rec
            (dy,) = tr.op(reads=[dy, mask], outs=[(net._nm("ddrop"), nbytes(B, *xs))])
        elif kind == "fc":
            _, x, din, name, dout = rec
            (net.grads[name + ".bias"],) = tr.op(reads=[dy], outs=[(net._nm("dfb"), nbytes(dout))])
            (net.grads[name + ".w"],) = tr.op(reads=[x, dy], outs=[(net._nm("dfw"), nbytes(din, dout))])
            (dy,) = tr.op(reads=[dy, ps.p[name + ".w"]], outs=[(net._nm("dfx"), nbytes(B, din))])
        elif kind == "add":
            stack.append(dy)       # the same gradient flows into both branches
        elif kind == "fork_main_done":
            # main branch finished: park its input gradient, continue with the skip branch
            skip_dy = stack.pop()
            stack.append(dy)
            dy = skip_dy
        elif kind == "fork":
            _, xs = rec
            main_dy = stack.pop()
            (dy,) = tr.op(reads=[dy, main_dy], outs=[(net._nm("dsum"), nbytes(B, *xs))])
        else:
            raise AssertionError(kind)


RESNET_STAGES = ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))


def resnet50_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    sh: List[Tuple[str, Tuple[int, ...]]] = [("conv1", (64, 3, 7, 7)), ("bn1.g", (64,)), ("bn1.b", (64,))]
    cin = 64
    for s, (w, blocks, _) in enumerate(RESNET_STAGES):
        for b in range(blocks):
            p = f"s{s}b{b}"
            for j, (ci, co, k) in enumerate(((cin, w, 1), (w, w, 3), (w, 4 * w, 1))):
                sh += [(f"{p}.c{j}", (co, ci, k, k)), (f"{p}.n{j}.g", (co,)), (f"{p}.n{j}.b", (co,))]
            if b == 0:
                sh += [(f"{p}.cd", (4 * w, cin, 1, 1)), (f"{p}.nd.g", (4 * w,)), (f"{p}.nd.b", (4 * w,))]
            cin = 4 * w
    sh += [("fc.w", (2048, 1000)), ("fc.bias", (1000,))]
    return sh


def resnet50_iteration(tr: Trace, ps: Params, batch: int, it: int, image: int = 224, fine_adam: bool = True) -> Params:
    net = _ConvNet(tr, ps, batch, it, workspace=True)
    x, y = tr.op(outs=[(f"i{it}.x", nbytes(batch, 3, image, image)), (f"i{it}.y", nbytes(batch))])
    h, hs = net.conv(x, (3, image, image), "conv1", 64, 7, 2)
    h = net.relu(net.bn(h, hs, "bn1"), hs)
    h, hs = net.pool(h, hs, 2)
    for s, (w, blocks, stride) in enumerate(RESNET_STAGES):
        for b in range(blocks):
            p = f"s{s}b{b}"
            st = stride if b == 0 else 1
            net.tape.append(("fork", hs))
            skip, skips = h, hs
            if b == 0:
                skip, skips = net.conv(h, hs, f"{p}.cd", 4 * w, 1, st)
                skip = net.bn(skip, skips, f"{p}.nd")
            net.tape.append(("fork_main_done",))
            m, ms = net.conv(h, hs, f"{p}.c0", w, 1, 1)
            m = net.relu(net.bn(m, ms, f"{p}.n0"), ms)
            m, ms = net.conv(m, ms, f"{p}.c1", w, 3, st)
            m = net.relu(net.bn(m, ms, f"{p}.n1"), ms)
            m, ms = net.conv(m, ms, f"{p}.c2", 4 * w, 1, 1)
            m = net.bn(m, ms, f"{p}.n2")
            h = net.relu(net.add(m, skip, ms), ms)
            hs = ms
    h, hs = net.pool(h, hs, hs[1])
    logits = net.fc(h, 2048, "fc", 1000)
    dy = net.loss(logits, y, 1000)
    _conv_backward(net, dy, {})
    return adam(tr, ps, net.grads, fine=fine_adam, it=it)


VGG16_CFG = (64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M")


def vgg16_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    sh: List[Tuple[str, Tuple[int, ...]]] = []
    cin, k = 3, 0
    for c in VGG16_CFG:
        if c == "M":
            continue
        sh += [(f"c{k}", (c, cin, 3, 3)), (f"c{k}.bias", (c,))]
        cin, k = c, k + 1
    for j, (di, do) in enumerate(((512 * 7 * 7, 4096), (4096, 4096), (4096, 1000))):
        sh += [(f"f{j}.w", (di, do)), (f"f{j}.bias", (do,))]
    return sh


def vgg16_iteration(tr: Trace, ps: Params, batch: int, it: int, image: int = 224, fine_adam: bool = True) -> Params:
    net = _ConvNet(tr, ps, batch, it, workspace=True)
    x, y = tr.op(outs=[(f"i{it}.x", nbytes(batch, 3, image, image)), (f"i{it}.y", nbytes(batch))])
    h, hs, k = x, (3, image, image), 0
    for c in VGG16_CFG:
        if c == "M":
            h, hs = net.pool(h, hs, 2)
        else:
            h, hs = net.conv(h, hs, f"c{k}", c, 3, 1)
            h = net.relu(net.bias(h, hs, f"c{k}.bias"), hs)
            k += 1
    din = prod(hs)
    for j, do in enumerate((4096, 4096, 1000)):
        h = net.fc(h, din, f"f{j}", do)
        if j < 2:
            h = net.dropout(net.relu(h, (do,)), (do,))
        din = do
    dy = net.loss(h, y, 1000)
    _conv_backward(net, dy, {})
    return adam(tr, ps, net.grads, fine=fine_adam, it=it)


# ----------------------------------------------------------------- transformer


def bert_shapes(layers: int = 12, hidden: int = 768, ffn: int = 3072, vocab: int = 30522, seq: int = 512):
    sh: List[Tuple[str, Tuple[int, ...]]] = [("emb.word", (vocab, hidden)), ("emb.pos", (seq, hidden)),
                                             ("emb.type", (2, hidden)), ("emb.ln.g", (hidden,)), ("emb.ln.b", (hidden,))]
    for l in range(layers):
        p = f"L{l}"
        for nm in ("q", "k", "v", "o"):
            sh += [(f"{p}.{nm}.w", (hidden, hidden)), (f"{p}.{nm}.bias", (hidden,))]
        sh += [(f"{p}.ln1.g", (hidden,)), (f"{p}.ln1.b", (hidden,)), (f"{p}.f1.w", (hidden, ffn)), (f"{p}.f1.bias", (ffn,)),
               (f"{p}.f2.w", (ffn, hidden)), (f"{p}.f2.bias", (hidden,)), (f"{p}.ln2.g", (hidden,)), (f"{p}.ln2.b", (hidden,))]
    sh += [("head.w", (hidden, hidden)), ("head.bias", (hidden,)), ("cls.w", (hidden, 2)), ("cls.bias", (2,))]
    return sh


def bert_iteration(tr: Trace, ps: Params, batch: int, it: int, layers: int = 12, hidden: int = 768, heads: int = 12,
                   ffn: int = 3072, seq: int = 512, fine_adam: bool = True) -> Params:
    """Encoder with per-head attention tensors (q, k, v, scores, probabilities,
    context are separate tensors per head, as a head-batched kernel sequence
    would produce them)."""
    t = f"i{it}"
    B, S, H, dh = batch, seq, hidden, hidden // heads
    act = nbytes(B, S, H)
    g: Dict[str, int] = {}
    op = tr.op
    ids, y = op(outs=[(f"{t}.ids", nbytes(B, S)), (f"{t}.y", nbytes(B))])
    (e,) = op(reads=[ids, ps.p["emb.word"], ps.p["emb.pos"], ps.p["emb.type"]], outs=[(f"{t}.emb", act)])
    h, e_mean, e_rstd = op(reads=[e, ps.p["emb.ln.g"], ps.p["emb.ln.b"]],
                           outs=[(f"{t}.embln", act), (f"{t}.embmu", nbytes(B, S)), (f"{t}.embrs", nbytes(B, S))])
    tape = []
    for l in range(layers):
        p = f"L{l}"
        n = f"{t}.{p}"
        x_in = h
        proj = {}
        for nm in ("q", "k", "v"):
            (proj[nm],) = op(reads=[x_in, ps.p[f"{p}.{nm}.w"], ps.p[f"{p}.{nm}.bias"]], outs=[(f"{n}.{nm}", act)])
        hq, hk, hv, hsc, hpr, hmask, hctx = [], [], [], [], [], [], []
        for a in range(heads):
            q_a, k_a, v_a = op(reads=[proj["q"], proj["k"], proj["v"]],
                               outs=[(f"{n}.q{a}", nbytes(B, S, dh)), (f"{n}.k{a}", nbytes(B, S, dh)), (f"{n}.v{a}", nbytes(B, S, dh))])
            (sc,) = op(reads=[q_a, k_a], outs=[(f"{n}.sc{a}", nbytes(B, S, S))])
            (sm,) = op(reads=[sc], outs=[(f"{n}.sm{a}", nbytes(B, S, S))])
            pr, mk = op(reads=[sm], outs=[(f"{n}.pr{a}", nbytes(B, S, S)), (f"{n}.pm{a}", nbytes(B, S, S) // 4)])
            (cx,) = op(reads=[pr, v_a], outs=[(f"{n}.cx{a}", nbytes(B, S, dh))])
            hq.append(q_a); hk.append(k_a); hv.append(v_a); hsc.append(sm); hpr.append(pr); hmask.append(mk); hctx.append(cx)
        (ctx,) = op(reads=hctx, outs=[(f"{n}.ctx", act)])
        (ao,) = op(reads=[ctx, ps.p[f"{p}.o.w"], ps.p[f"{p}.o.bias"]], outs=[(f"{n}.ao", act)])
        ad, adm = op(reads=[ao], outs=[(f"{n}.aod", act), (f"{n}.aom", act // 4)])
        (r1,) = op(reads=[ad, x_in], outs=[(f"{n}.r1", act)])
        l1, mu1, rs1 = op(reads=[r1, ps.p[f"{p}.ln1.g"], ps.p[f"{p}.ln1.b"]],
                          outs=[(f"{n}.ln1", act), (f"{n}.mu1", nbytes(B, S)), (f"{n}.rs1", nbytes(B, S))])
        (f1,) = op(reads=[l1, ps.p[f"{p}.f1.w"], ps.p[f"{p}.f1.bias"]], outs=[(f"{n}.f1", nbytes(B, S, ffn))])
        (ge,) = op(reads=[f1], outs=[(f"{n}.gelu", nbytes(B, S, ffn))])
        (f2,) = op(reads=[ge, ps.p[f"{p}.f2.w"], ps.p[f"{p}.f2.bias"]], outs=[(f"{n}.f2", act)])
        fd, fdm = op(reads=[f2], outs=[(f"{n}.f2d", act), (f"{n}.f2m", act // 4)])
        (r2,) = op(reads=[fd, l1], outs=[(f"{n}.r2", act)])
        h, mu2, rs2 = op(reads=[r2, ps.p[f"{p}.ln2.g"], ps.p[f"{p}.ln2.b"]],
                         outs=[(f"{n}.ln2", act), (f"{n}.mu2", nbytes(B, S)), (f"{n}.rs2", nbytes(B, S))])
        tape.append(dict(p=p, n=n, x_in=x_in, proj=proj, hq=hq, hk=hk, hv=hv, hsm=hsc, hpr=hpr, hmask=hmask, ctx=ctx, adm=adm,
                         r1=r1, mu1=mu1, rs1=rs1, l1=l1, f1=f1, ge=ge, fdm=fdm, r2=r2, mu2=mu2, rs2=rs2))
    (pooled,) = op(reads=[h, ps.p["head.w"], ps.p["head.bias"]], outs=[(f"{t}.pooled", nbytes(B, H))])
    (logits,) = op(reads=[pooled, ps.p["cls.w"], ps.p["cls.bias"]], outs=[(f"{t}.logits", nbytes(B, 2))])
    probs, loss = op(reads=[logits, y], outs=[(f"{t}.probs", nbytes(B, 2)), (f"{t}.loss", F32)])
    # backward
    (dlog,) = op(reads=[probs, y, loss], outs=[(f"{t}.dlogits", nbytes(B, 2))])
    g["cls.w"], g["cls.bias"], dpool = op(reads=[dlog, pooled, ps.p["cls.w"]],
                                          outs=[(f"{t}.dclsw", nbytes(H, 2)), (f"{t}.dclsb", nbytes(2)), (f"{t}.dpooled", nbytes(B, H))])
    g["head.w"], g["head.bias"], dh_ = op(reads=[dpool, h, pooled, ps.p["head.w"]],
                                          outs=[(f"{t}.dheadw", nbytes(H, H)), (f"{t}.dheadb", nbytes(H)), (f"{t}.dh", act)])
    for rec in reversed(tape):
        p, n = rec["p"], rec["n"]
        dr2, g[f"{p}.ln2.g"], g[f"{p}.ln2.b"] = op(reads=[dh_, rec["r2"], rec["mu2"], rec["rs2"], ps.p[f"{p}.ln2.g"]],
                                                   outs=[(f"{n}.dr2", act), (f"{n}.dln2g", nbytes(H)), (f"{n}.dln2b", nbytes(H))])
        (dfd,) = op(reads=[dr2, rec["fdm"]], outs=[(f"{n}.df2d", act)])
        g[f"{p}.f2.w"], g[f"{p}.f2.bias"] = op(reads=[dfd, rec["ge"]], outs=[(f"{n}.df2w", nbytes(ffn, H)), (f"{n}.df2b", nbytes(H))])
        (dge,) = op(reads=[dfd, ps.p[f"{p}.f2.w"]], outs=[(f"{n}.dgelu", nbytes(B, S, ffn))])
        (df1,) = op(reads=[dge, rec["f1"]], outs=[(f"{n}.df1", nbytes(B, S, ffn))])
        g[f"{p}.f1.w"], g[f"{p}.f1.bias"] = op(reads=[df1, rec["l1"]], outs=[(f"{n}.df1w", nbytes(H, ffn)), (f"{n}.df1b", nbytes(ffn))])
        (dl1a,) = op(reads=[df1, ps.p[f"{p}.f1.w"]], outs=[(f"{n}.dl1a", act)])
        (dl1,) = op(reads=[dl1a, dr2], outs=[(f"{n}.dl1", act)])
        dr1, g[f"{p}.ln1.g"], g[f"{p}.ln1.b"] = op(reads=[dl1, rec["r1"], rec["mu1"], rec["rs1"], ps.p[f"{p}.ln1.g"]],
                                                   outs=[(f"{n}.dr1", act), (f"{n}.dln1g", nbytes(H)), (f"{n}.dln1b", nbytes(H))])
        (dad,) = op(reads=[dr1, rec["adm"]], outs=[(f"{n}.dao", act)])
        g[f"{p}.o.w"], g[f"{p}.o.bias"] = op(reads=[dad, rec["ctx"]], outs=[(f"{n}.dow", nbytes(H, H)), (f"{n}.dob", nbytes(H))])
        (dctx,) = op(reads=[dad, ps.p[f"{p}.o.w"]], outs=[(f"{n}.dctx", act)])
        dq, dk, dv = [], [], []
        for a in range(heads):
            dpr, dv_a = op(reads=[dctx, rec["hv"][a], rec["hpr"][a]],
                           outs=[(f"{n}.dpr{a}", nbytes(B, S, S)), (f"{n}.dv{a}", nbytes(B, S, dh))])
            (dsm,) = op(reads=[dpr, rec["hmask"][a]], outs=[(f"{n}.dsm{a}", nbytes(B, S, S))])
            (dsc,) = op(reads=[dsm, rec["hsm"][a]], outs=[(f"{n}.dsc{a}", nbytes(B, S, S))])
            dq_a, dk_a = op(reads=[dsc, rec["hq"][a], rec["hk"][a]],
                            outs=[(f"{n}.dq{a}", nbytes(B, S, dh)), (f"{n}.dk{a}", nbytes(B, S, dh))])
            dq.append(dq_a); dk.append(dk_a); dv.append(dv_a)
        dxs = []
        for nm, parts in (("q", dq), ("k", dk), ("v", dv)):
            (dp,) = op(reads=parts, outs=[(f"{n}.d{nm}", act)])
            g[f"{p}.{nm}.w"], g[f"{p}.{nm}.bias"] = op(reads=[dp, rec["x_in"]], outs=[(f"{n}.d{nm}w", nbytes(H, H)), (f"{n}.d{nm}b", nbytes(H))])
            (dx,) = op(reads=[dp, ps.p[f"{p}.{nm}.w"]], outs=[(f"{n}.dx{nm}", act)])
            dxs.append(dx)
        (dh_,) = op(reads=[*dxs, dr1], outs=[(f"{n}.dx", act)])
    de, g["emb.ln.g"], g["emb.ln.b"] = op(reads=[dh_, e, e_mean, e_rstd, ps.p["emb.ln.g"]],
                                          outs=[(f"{t}.demb", act), (f"{t}.dembg", nbytes(H)), (f"{t}.dembb", nbytes(H))])
    g["emb.word"], g["emb.pos"], g["emb.type"] = op(reads=[de, ids], outs=[(f"{t}.dword", nbytes(*ps.shape["emb.word"])),
                                                                           (f"{t}.dpos", nbytes(*ps.shape["emb.pos"])),
                                                                           (f"{t}.dtype", nbytes(*ps.shape["emb.type"]))])
    return adam(tr, ps, g, fine=fine_adam, it=it)
