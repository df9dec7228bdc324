"""Gradient noise per layer of each stochastic gradient method (Section 4.3, the figure on gradient noise): the full
gradient over a training set is computed once, then each method's estimate on single minibatches is compared
with it, and the mean squared deviation is reported layer by layer.  Methods: the baseline minibatch, RAD with
the same sample for every example, RAD with a different sample per example, a reduced minibatch of about the
same memory, and RAD on a larger minibatch.

The training set is synthetic (seeded, the shapes and value statistics of the paper's datasets, which are not
available here); everything is computed by rad_train_step through the C ABI.

    python -m paper_2007_10412_amd.gradient_noise --arch cnn --train 1200 --draws 16      (or --arch mlp, --arch rnn)

prints one JSON object.  `measure` takes the step function as an argument, so that a test can run the same
procedure on another implementation of the step."""
import argparse
import json

import numpy as np


def paper_arch(arch):
    """Appendix A, architectures used."""
    if arch == "mlp":
        return dict(kind="mlp", dims=(784, 300, 300, 300, 10), batch=150, reduced=22)
    if arch == "rnn":      # reduced minibatch of 21 (Appendix A, RNN training details)
        return dict(kind="rnn", T=784, d_input=1, hidden=100, classes=10, batch=150, reduced=21)
    return dict(kind="cnn", channels=(3, 16, 32, 32, 32), pool=(0, 2, 0, 2), ksize=5, hw=32, classes=10, batch=150,
                reduced=20)


def methods_for(cfg, p):
    """name -> (minibatch size, scheme, fraction); scheme numbers are rad_scheme's."""
    b = cfg["batch"]
    return {"baseline": (b, 0, 1.0), "same_sample": (b, 2, p), "different_sample": (b, 3, p),
            "reduced_batch": (cfg["reduced"], 0, 1.0), "different_sample_2x_batch": (2 * b, 3, p)}


def measure(step, n_train, methods, draws, seed=0):
    """step(first, count, scheme, p, sample_seed) -> list of per-layer gradient arrays of the minibatch
    [first, first + count) (mean loss over the minibatch).  Returns {method: [mse per layer]}.

    The full gradient is the average of the exact minibatch gradients over the whole set, taken in chunks of
    the baseline size (n_train must be a multiple of it).  Draw i of a method uses the minibatch starting at a
    seeded random offset (a multiple of the method's size) and the sampling seed i + 1."""
    base = methods["baseline"][0]
    assert n_train % base == 0
    full = None
    for first in range(0, n_train, base):
        g = step(first, base, 0, 1.0, 0)
        full = [np.asarray(a, np.float64).copy() for a in g] if full is None else [f + a for f, a in zip(full, g)]
    full = [f / (n_train // base) for f in full]
    out = {}
    for name, (size, scheme, p) in methods.items():
        rng = np.random.default_rng(seed)
        acc = [0.0] * len(full)
        for i in range(draws):
            first = int(rng.integers(0, n_train // size)) * size
            g = step(first, size, scheme, p, i + 1)
            for l, (a, f) in enumerate(zip(g, full)):
                acc[l] += float(np.mean((np.asarray(a, np.float64) - f) ** 2))
        out[name] = [a / draws for a in acc]
    return out


class GpuStep:
    """rad_train_step on slices of a device-resident training set; one model per (size, scheme, p)."""

    def __init__(self, cfg, data):
        import torch
        from . import binding as B
        self.B, self.torch, self.cfg = B, torch, cfg
        self.ctx = B.rad_ctx_create()
        self.x = torch.from_numpy(data["x"]).cuda()
        self.labels = torch.from_numpy(data["labels"]).cuda()
        if cfg["kind"] == "mlp":
            ws = [a for pair in zip(data["Ws"], data["bs"]) for a in pair]
            self.weight_slots = list(range(0, len(ws), 2))
        elif cfg["kind"] == "rnn":      # "layers" of the recurrent model: input, recurrent and output weights
            ws = [data[n] for n in ("W_ih", "W_hh", "b", "W_ho", "b_o")]
            self.weight_slots = [0, 1, 3]
        else:
            ws = [a for cv in data["convs"] for a in (cv["W"], cv["b"])] + [data["fc"][0], data["fc"][1]]
            self.weight_slots = list(range(0, len(ws), 2))
        self.params = [torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in ws]
        self.grads = [torch.empty_like(a) for a in self.params]
        self.models = {}

    def model(self, size, scheme, p):
        key = (size, scheme, p)
        if key not in self.models:
            B, c = self.B, self.cfg
            if c["kind"] == "mlp":
                self.models[key] = B.rad_model_create_mlp(self.ctx, B.RAD_F32, size, list(c["dims"]), True, scheme, p)
            elif c["kind"] == "rnn":
                self.models[key] = B.rad_model_create_rnn(self.ctx, size, c["T"], c["d_input"], c["hidden"], c["classes"],
                                                          scheme, p)
            else:
                self.models[key] = B.rad_model_create_cnn(self.ctx, size, list(c["channels"]), list(c["pool"]), c["ksize"],
                                                          c["hw"], c["hw"], c["classes"], scheme, p)
        return self.models[key]

    def __call__(self, first, count, scheme, p, sample_seed):
        B = self.B
        B.rad_train_step(self.ctx, self.model(count, scheme, p), B.make_sampling(scheme, p, sample_seed, 0, 0),
                         self.x[first:first + count], self.labels[first:first + count], self.params, self.grads)
        return [self.grads[i].cpu().numpy() for i in self.weight_slots]

    def close(self):
        for m in self.models.values():
            self.B.rad_model_destroy(m)
        self.B.rad_ctx_destroy(self.ctx)


def training_set(cfg, n_train, seed=1234):
    from . import synth
    if cfg["kind"] == "mlp":
        return synth.mlp(seed=seed, batch=n_train, dims=cfg["dims"], bias_scale=0.0)
    if cfg["kind"] == "rnn":
        return synth.rnn(seed=seed, batch=n_train, T=cfg["T"], d_input=cfg["d_input"], hidden=cfg["hidden"],
                         classes=cfg["classes"], identity=True)
    return synth.cnn(seed=seed, batch=n_train, channels=cfg["channels"], pool=cfg["pool"], ksize=cfg["ksize"],
                     hw=cfg["hw"], classes=cfg["classes"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--arch", default="cnn", choices=["cnn", "mlp", "rnn"])
    ap.add_argument("--train", type=int, default=1200, help="training-set size (a multiple of 300)")
    ap.add_argument("--draws", type=int, default=16)
    ap.add_argument("--p", type=float, default=0.1)
    args = ap.parse_args()
    cfg = paper_arch(args.arch)
    if args.train % (2 * cfg["batch"]):
        raise SystemExit("--train must be a multiple of %d" % (2 * cfg["batch"]))
    step = GpuStep(cfg, training_set(cfg, args.train))
    try:
        res = measure(step, args.train, methods_for(cfg, args.p), args.draws)
    finally:
        step.close()
    print(json.dumps({"arch": args.arch, "train": args.train, "draws": args.draws, "p": args.p,
                      "mse_per_layer": res}))


if __name__ == "__main__":
    main()
