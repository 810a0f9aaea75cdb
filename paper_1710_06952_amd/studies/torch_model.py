"""AD-PSGD for a model the library does not know: the gradient step of Algorithm 1 is PyTorch autograd,
everything else (sampling of workers and neighbours, stale reads, atomic pairwise averaging, the update
with momentum and weight decay, packing of the events into conflict-free rounds) stays in the library
(model "external", adpsgd_run_events_with).

The n replicas of the network live as the rows of the engine's n x d matrix; for every event the library
hands the gradient function the row to evaluate at (as stale as the schedule says) and the slot that
receives the gradient.  The function below views the row as the parameters of a torch.nn.Module
(torch.func.functional_call), draws the event's minibatch from the worker's local data with a generator
seeded by the event number, and lets autograd write the flattened gradient.

By default the run uses the wait-free variant (a worker evaluates its next gradient at its stale copy with
its own pending gradient applied), the form the paper's implementation takes.  The example network is a small classifier with a normalisation layer and a tanh hidden layer, on the
Gaussian mixture of the convergence study; any module whose parameters are fp32 works the same way.

    python -m paper_1710_06952_amd.studies.torch_model [--n 8] [--epochs 4] [--json]
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from .convergence import make_problem, ring


def build_module(din, hidden, classes):
    import torch
    return torch.nn.Sequential(torch.nn.Linear(din, hidden), torch.nn.LayerNorm(hidden), torch.nn.Tanh(),
                               torch.nn.Linear(hidden, classes))


class FlatModule:
    """A module evaluated at a flat parameter vector (views, no copies)."""

    def __init__(self, module):
        self.module = module
        self.shapes = [(name, p.shape, p.numel()) for name, p in module.named_parameters()]
        self.d = sum(c for _, _, c in self.shapes)

    def flatten_initial(self):
        import torch
        return torch.cat([p.detach().reshape(-1) for p in self.module.parameters()]).float().cpu().numpy()

    def unflatten(self, x):
        out, at = {}, 0
        for name, shape, count in self.shapes:
            out[name] = x[at:at + count].view(shape)
            at += count
        return out

    def loss_and_gradient(self, x, inputs, labels, out):
        """Cross-entropy of the module at parameters x on (inputs, labels); the gradient goes to `out`."""
        import torch
        xr = x.detach().clone().requires_grad_(True)
        logits = torch.func.functional_call(self.module, self.unflatten(xr), (inputs,))
        loss = torch.nn.functional.cross_entropy(logits, labels)
        (grad,) = torch.autograd.grad(loss, xr)
        out.copy_(grad)
        return loss

    def evaluate(self, x, inputs, labels):
        import torch
        with torch.no_grad():
            logits = torch.func.functional_call(self.module, self.unflatten(x), (inputs,))
            return (float(torch.nn.functional.cross_entropy(logits, labels)),
                    float((logits.argmax(1) != labels).float().mean()))


def run_study(n=8, dims=(32, 64, 6), rows=1024, M=32, epochs=4, T_max=3, gamma=0.05, momentum=0.9, weight_decay=1e-4,
              seed=0, device="cuda:0", wait_free=True):
    import torch
    from .. import Engine, adpsgd_make_schedule
    torch.manual_seed(seed)
    flat = FlatModule(build_module(*dims).to(device))
    feats, labels, _ = make_problem(n, rows, dims, seed)
    X = [torch.from_numpy(f).to(device) for f in feats]
    Y = [torch.from_numpy(y).to(device).long() for y in labels]
    allX, allY = torch.cat(X), torch.cat(Y)
    eng = Engine(ring(n), flat.d, "external", gamma=gamma, T_max=T_max, momentum=momentum, weight_decay=weight_decay,
                 local_compensation=wait_free, device=device)
    eng.set_models(flat.flatten_initial())
    events_per_epoch = n * rows // M

    def gradient(worker, event, xhat, out):
        gen = torch.Generator(device=device)
        gen.manual_seed(seed * 1_000_003 + event)
        idx = torch.randint(0, rows, (M,), device=device, generator=gen)
        flat.loss_and_gradient(xhat, X[worker][idx], Y[worker][idx], out)

    mean = lambda: torch.from_numpy(eng.get_mean_model()).to(device)
    curve = [flat.evaluate(mean(), allX, allY)]
    sched = adpsgd_make_schedule(ring(n), epochs * events_per_epoch, seed=seed, T_max=T_max)
    # an epoch per call; the calls look ahead, so staleness reaches across the epochs as in one long call
    eng.run_events_in_pieces(sched, events_per_epoch, gradient_fn=gradient,
                             between=lambda _events: curve.append(flat.evaluate(mean(), allX, allY)))
    res = {"n": n, "d": flat.d, "rows": rows, "M": M, "epochs": epochs, "T_max": T_max, "gamma": gamma,
           "momentum": momentum, "weight_decay": weight_decay, "loss": [c[0] for c in curve], "error": [c[1] for c in curve],
           "consensus_distance": eng.consensus_distance(), "rounds": eng.get_stats()["rounds"],
           "events": eng.get_stats()["events"]}
    eng.close()
    return res


def format_table(res):
    lines = ["epoch |     loss |  error", "-" * 26]
    for e, (l, r) in enumerate(zip(res["loss"], res["error"])):
        lines.append("%5d | %8.5f | %6.4f" % (e, l, r))
    lines.append("%d events in %d rounds; consensus distance %.3g" % (res["events"], res["rounds"], res["consensus_distance"]))
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--n", type=int, default=8)
    ap.add_argument("--epochs", type=int, default=4)
    ap.add_argument("--gamma", type=float, default=0.05)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args(argv)
    res = run_study(a.n, epochs=a.epochs, gamma=a.gamma, seed=a.seed)
    print(json.dumps(res) if a.json else format_table(res))


if __name__ == "__main__":
    main()
