"""Device-memory plumbing around the C-ABI handle: PyTorch allocates the model
matrix, the pending-gradient workspace and the workers' data on the GPU and
lends a stream; every computation happens inside libadpsgd.so."""
from __future__ import annotations

import numpy as np

from . import binding as B

_MODELS = {"lsq": B.MODEL_LSQ, "logreg": B.MODEL_LOGREG, "synth": B.MODEL_SYNTH, "mlp": B.MODEL_MLP,
           "external": B.MODEL_EXTERNAL}


def _pad(d, mult=64):
    return (d + mult - 1) // mult * mult


class _DeviceSpan:
    """d fp32 values at a device address, for torch.as_tensor (no copy)."""

    def __init__(self, ptr, d):
        self.__cuda_array_interface__ = {"shape": (d,), "typestr": "<f4", "data": (ptr, False), "version": 2}


def _device_vector(torch, ptr, d, device):
    return torch.as_tensor(_DeviceSpan(ptr, d), device=device)


class Engine:
    def __init__(self, graph, d, model, *, M=0, gamma=0.0, lam=0.0, grad_sum=False, T_max=0, synth_std=0.0,
                 synth_seed=0, mlp=(0, 0, 0), n_slots=None, profile=False, momentum=0.0, weight_decay=0.0,
                 local_compensation=False, dense_gradient=False, verify_plan=False, sync_in_place=False, device="cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("Engine needs a GPU: the HIP library is the only implementation")
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.n = len(graph[0]) - 1
        self.d = d
        self.ld = _pad(d)
        self.model = _MODELS[model] if isinstance(model, str) else model
        self.M = M
        self.T_max = T_max
        self.X = torch.zeros((self.n, self.ld), dtype=torch.float32, device=self.device)
        self.Xbf16 = None
        self.workspace = None
        ws_ptr, ws_bytes = None, 0
        if self.model != B.MODEL_SYNTH:
            if n_slots is None:
                n_slots = max(T_max + 1, min(4 * self.n, 256))
                budget = 8 << 30                         # keep the slots within 8 GiB by default
                n_slots = max(T_max + 1, min(n_slots, budget // (self.ld * 4)))
            self.workspace = torch.empty((n_slots, self.ld), dtype=torch.float32, device=self.device)
            ws_ptr, ws_bytes = self.workspace.data_ptr(), n_slots * self.ld * 4
        if self.model == B.MODEL_MLP:
            self.Xbf16 = torch.zeros((self.n, self.ld), dtype=torch.bfloat16, device=self.device)
        self.V = None
        if momentum != 0.0 or weight_decay != 0.0:
            self.V = torch.zeros((self.n, self.ld), dtype=torch.float32, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.h = B.Handle(graph, d, model=self.model, X_ptr=self.X.data_ptr(), ldx=self.ld, M=M, gamma=gamma,
                          lam=lam, grad_sum=grad_sum, T_max=T_max, synth_std=synth_std, synth_seed=synth_seed,
                          mlp=mlp, Xbf16_ptr=None if self.Xbf16 is None else self.Xbf16.data_ptr(),
                          workspace_ptr=ws_ptr, workspace_bytes=ws_bytes, stream=self.stream.cuda_stream,
                          flags=(B.FLAG_PROFILE if profile else 0) | (B.FLAG_DENSE_GRADIENT if dense_gradient else 0) |
                          (B.FLAG_VERIFY_PLAN if verify_plan else 0) | (B.FLAG_SYNC_IN_PLACE if sync_in_place else 0), momentum=momentum, weight_decay=weight_decay,
                          V_ptr=None if self.V is None else self.V.data_ptr(),
                          local_compensation=local_compensation)
        self._data = []
        self.loss = None

    def load_data(self, features, targets):
        """features/targets: per-worker numpy arrays (host) or torch tensors already on the GPU."""
        torch = self.torch
        for i, (f, t) in enumerate(zip(features, targets)):
            if isinstance(f, np.ndarray):
                rows, cols = f.shape
                mult = 8 if f.dtype == np.uint16 else 4
                ld = _pad(cols, mult)
                if f.dtype == np.uint16:
                    ft = torch.zeros((rows, ld), dtype=torch.bfloat16, device=self.device)
                    ft[:, :cols] = torch.from_numpy(f.view(np.int16)).to(self.device).view(torch.bfloat16)
                else:
                    ft = torch.zeros((rows, ld), dtype=torch.float32, device=self.device)
                    ft[:, :cols] = torch.from_numpy(f).to(self.device)
                tt = torch.from_numpy(np.ascontiguousarray(t)).to(self.device)
            else:
                ft, tt = f, t
                rows, ld = ft.shape[0], ft.stride(0)
            self._data.append((ft, tt))
            self.h.load_data(i, ft.data_ptr(), rows, ld, tt.data_ptr())
        torch.cuda.synchronize(self.device)

    def set_models(self, x, broadcast=True):
        x = np.ascontiguousarray(x, dtype=np.float32)
        self.h.set_models(x, 0 if broadcast else x.shape[1])

    def run_events(self, schedule, want_loss=False):
        loss_ptr = None
        if want_loss:
            self.loss = self.torch.zeros(len(schedule["worker"]), dtype=self.torch.float32, device=self.device)
            loss_ptr = self.loss.data_ptr()
        self.h.run_events(schedule, loss_ptr)

    def run_events_in_pieces(self, schedule, piece, between=None, gradient_fn=None):
        """A long schedule as calls of ``piece`` events, each looking T_max events ahead, so that staleness
        reaches across the cuts and the result is that of a single call.  ``between(events_applied)`` runs
        after every call (logging, diagnostics).  gradient_fn: as in run_events_with, for model "external";
        it is handed event numbers that count from the start of ``schedule``."""
        K = len(schedule["worker"])
        look = 0 if self.model == B.MODEL_SYNTH else self.T_max
        extra = schedule.get("extra_pairs")
        for a in range(0, K, piece):
            b = min(a + piece, K)
            end = min(b + look, K)
            part = {k: (None if schedule.get(k) is None else schedule[k][a:end])
                    for k in ("worker", "neighbour", "tau", "batch_idx", "gamma")}
            if extra is not None:
                ptr = np.asarray(extra[0], dtype=np.int64)
                part["extra_pairs"] = (ptr[a:end + 1] - ptr[a], extra[1][ptr[a]:ptr[end]], extra[2][ptr[a]:ptr[end]])
            part["lookahead"] = end - b
            if gradient_fn is None:
                self.run_events(part)
            else:
                self.run_events_with(part, lambda worker, event, xhat, g, a=a: gradient_fn(worker, a + event, xhat, g))
            if between is not None:
                between(b)

    def _per_group(self, gradient_fn):
        """Wraps gradient_fn(worker, event, xhat, g), which takes two views of device memory, into the
        binding's form (a list of requests with raw pointers)."""
        ws, ld, d = self.workspace.view(-1, self.ld), self.ld, self.d
        x_base, w_base = self.X.data_ptr(), self.workspace.data_ptr()

        def per_group(requests, _stream):
            for worker, event, xhat_ptr, g_ptr in requests:
                if xhat_ptr == x_base + worker * ld * 4:
                    xhat = self.X[worker, :d]
                else:                       # wait-free variant: a compensated copy in the library's scratch memory
                    xhat = _device_vector(self.torch, xhat_ptr, d, self.device)
                gradient_fn(worker, event, xhat, ws[(g_ptr - w_base) // (ld * 4), :d])

        return per_group

    def run_events_with(self, schedule, gradient_fn):
        """Model "external": gradient_fn(worker, event, xhat, g) is called for every event with two views
        of device memory, the model to evaluate at (d floats, read only) and the slot that receives the
        gradient; it must work on PyTorch's current stream, which is the stream the engine was created on."""
        self.h.run_events_with(schedule, self._per_group(gradient_fn))

    def run_sync_steps_with(self, steps, gradient_fn, gamma=None, weights=None):
        """Model "external": the synchronous comparison schedule; event = iteration * n + worker."""
        self.h.run_sync_steps_with(steps, self._per_group(gradient_fn), gamma, weights)

    def run_sync_steps(self, steps, batch_idx=None, gamma=None, weights=None, want_loss=False):
        """The synchronous comparison schedule (all workers step together, mixing with all neighbours)."""
        loss_ptr = None
        if want_loss:
            self.loss = self.torch.zeros(steps * self.n, dtype=self.torch.float32, device=self.device)
            loss_ptr = self.loss.data_ptr()
        self.h.run_sync_steps(steps, batch_idx, gamma, weights, loss_ptr)

    def get_loss(self):
        self.torch.cuda.synchronize(self.device)
        return self.loss.cpu().numpy()

    def get_models(self):
        return self.h.get_models()

    def get_bf16_models(self):
        return self.h.get_bf16_models()

    def get_momentum(self):
        return self.h.get_momentum()

    def get_mean_model(self):
        return self.h.get_mean_model()

    def consensus_distance(self, p=None):
        return self.h.consensus_distance(p)

    def objective(self, x=None, p=None):
        """The objective over all local data at x (numpy vector or None = the mean model), the workers
        weighted equally or by the probabilities p."""
        if x is None:
            return self.h.objective(None, p)
        xt = self.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
        return self.h.objective(xt.data_ptr(), p)

    def classification_error(self, x=None):
        """Fraction of the local samples misclassified at x (numpy vector or None = the mean model)."""
        if x is None:
            return self.h.classification_error(None)
        xt = self.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
        return self.h.classification_error(xt.data_ptr())

    def count_nonfinite(self):
        return self.h.count_nonfinite()

    def get_stats(self):
        return self.h.get_stats()

    def close(self):
        self.h.destroy()
