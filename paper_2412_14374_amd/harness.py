"""Device-memory plumbing around the C-ABI library for tests, smoke and the benchmark.

PyTorch is used for what it is good at here: allocating HBM, moving host arrays in and
out, and providing HIP streams.  Nothing in this file computes any part of the method.
"""
import numpy as np
import torch

from . import binding as B
from . import inputs as inp


def torch_dtype(w):
    return torch.bfloat16 if w.dtype == inp.DT_BF16 else torch.float32


def to_device(a, w, dev="cuda:0"):
    """float64 host array (already on the storage grid) -> device tensor of the storage dtype."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(torch_dtype(w)).contiguous()


def to_host(t):
    return t.detach().to(torch.float64).cpu().numpy()


class Stage:
    """Owns the arena and boundary tensors of one jpp_stage."""

    def __init__(self, w, max_in_flight=None, tasks=None, dev="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the stage executor only runs on a HIP device")
        self.w, self.dev = w, dev
        self.cfg = B.make_config(w)
        self.M = w.n_microbatches
        self.tasks = tasks if tasks is not None else default_tasks(w)
        peak = B.jpp_schedule_validate(self.cfg, self.M, self.tasks)
        # one slot above the schedule's peak lets the next forward's input be prefetched
        # (with weight-gradient groups a prefetch may open a group: one group's worth above it)
        self.max_in_flight = max_in_flight if max_in_flight is not None else peak + max(1, self.cfg.wgrad_group)
        nbytes = B.jpp_stage_arena_bytes(self.cfg, self.M, self.max_in_flight)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.h = B.jpp_stage_create(self.cfg, self.M, self.max_in_flight, base, nbytes)
        self.info = B.jpp_stage_param_info(self.h)
        self.pcount = B.jpp_stage_param_count(self.h)
        self.compute = torch.cuda.Stream(device=dev)
        self.side = torch.cuda.Stream(device=dev)
        self.V = len(w.stage_ids)
        self._keep = []

    def close(self):
        if self.h is not None:
            B.jpp_stage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- parameters ---------------------------------------------------------------------
    def layer_shapes(self):
        """(name, shape) per layer and for the head, as the library lays them out."""
        layer, head = [], []
        for name, shp, _ in self.info:
            if name.startswith("layer0."):
                layer.append((name.split(".", 1)[1], shp))
            elif name.startswith("head."):
                head.append((name.split(".", 1)[1], shp))
        return layer, head

    def pack_params(self, p):
        """p: {'layers': [dict], 'head': dict} of float64 arrays -> flat float32 host array."""
        flat = np.zeros(self.pcount, dtype=np.float32)
        for name, shp, off in self.info:
            grp, key = name.split(".", 1)
            if grp in ("head", "embed") and grp not in p:
                continue            # a virtual stage without the head / the embedding: its slots stay zero
            a = p[grp][key] if grp in ("head", "embed") else p["layers"][int(grp[5:])][key]
            assert tuple(a.shape) == tuple(shp), (name, a.shape, shp)
            flat[off:off + a.size] = a.reshape(-1)
        return flat

    def unpack_grads(self, flat):
        out = {"layers": [dict() for _ in range(self.w.n_layers)]}
        if self.w.loss_head:
            out["head"] = {}
        if getattr(self.w, "embed", 0):
            out["embed"] = {}
        for name, shp, off in self.info:
            grp, key = name.split(".", 1)
            a = flat[off:off + int(np.prod(shp))].reshape(shp)
            if grp in ("head", "embed"):
                out[grp][key] = a
            else:
                out["layers"][int(grp[5:])][key] = a
        return out

    def set_params_host(self, params_by_stage):
        for v, s in enumerate(self.w.stage_ids):
            flat = torch.from_numpy(self.pack_params(params_by_stage[s])).to(self.dev).to(torch_dtype(self.w))
            torch.cuda.synchronize()
            B.jpp_stage_set_params(self.h, v, flat.data_ptr(), True)

    def set_params_random(self, seed=0):
        """Fills parameters on the device (benchmark path): N(0, w_std) matrices, unit gains."""
        g = torch.Generator(device=self.dev)
        g.manual_seed(seed)
        for v in range(self.V):
            flat = torch.zeros(self.pcount, dtype=torch.float32, device=self.dev)
            for name, shp, off in self.info:
                n = int(np.prod(shp))
                if len(shp) == 2:
                    flat[off:off + n] = torch.randn(n, generator=g, device=self.dev) * self.w.w_std
                elif name.endswith("_g"):
                    flat[off:off + n] = 1.0
            flat = flat.to(torch_dtype(self.w))
            torch.cuda.synchronize()
            B.jpp_stage_set_params(self.h, v, flat.data_ptr(), True)
            del flat

    # ---- boundary -----------------------------------------------------------------------
    def bind(self, x=None, cot=None, targets=None, seed=1):
        """x, cot: {stage: [M arrays]} host float64 (or None: random on device)."""
        w, M, dt = self.w, self.M, torch_dtype(self.w)
        shp = (w.microbatch, w.seq_len, w.d_model)
        g = torch.Generator(device=self.dev)
        g.manual_seed(seed)
        self.in_x, self.in_c, self.out_y, self.out_dx, self.tg = [], [], [], [], []
        for v, s in enumerate(w.stage_ids):
            for i in range(M):
                if getattr(w, "embed", 0) and v == 0:
                    # the embedding stage reads int32 token ids
                    if x is not None:
                        self.in_x.append(torch.from_numpy(np.ascontiguousarray(x[s][i], dtype=np.int32)).to(self.dev))
                    else:
                        self.in_x.append(torch.randint(0, w.vocab, (w.microbatch, w.seq_len), generator=g,
                                                       device=self.dev, dtype=torch.int32))
                elif x is not None:
                    self.in_x.append(to_device(x[s][i], w, self.dev))
                else:
                    self.in_x.append(torch.randn(shp, generator=g, device=self.dev).to(dt))
                if not w.loss_head:
                    if cot is not None:
                        self.in_c.append(to_device(cot[s][i], w, self.dev))
                    else:
                        self.in_c.append((torch.randn(shp, generator=g, device=self.dev) * w.cot_std).to(dt))
                    self.out_y.append(torch.zeros(shp, dtype=dt, device=self.dev))
                else:
                    if targets is not None:
                        self.tg.append(torch.from_numpy(np.ascontiguousarray(targets[i], dtype=np.int32)).to(self.dev))
                    else:
                        self.tg.append(torch.randint(0, w.vocab, (w.microbatch, w.seq_len), generator=g,
                                                     device=self.dev, dtype=torch.int32))
                self.out_dx.append(torch.zeros(shp, dtype=dt, device=self.dev))
        torch.cuda.synchronize()
        ptrs = lambda ts: [t.data_ptr() for t in ts] if ts else None
        B.jpp_stage_bind_boundary(self.h, ptrs(self.in_x), ptrs(self.in_c), ptrs(self.out_y), ptrs(self.out_dx),
                                  ptrs(self.tg))

    # ---- execution ----------------------------------------------------------------------
    def zero_grads(self):
        B.jpp_stage_zero_grads(self.h, self.compute.cuda_stream)

    def run(self, tasks=None):
        arr, n = B.tasks_array(self.tasks if tasks is None else tasks)
        B.jpp_stage_run(self.h, arr, n, self.compute.cuda_stream, self.side.cuda_stream)

    def sync(self):
        self.compute.synchronize()
        self.side.synchronize()

    def grads_tensor(self, v):
        """fp32 device tensor copy of local virtual stage v's flat gradient buffer."""
        ptr, n = B.jpp_stage_grads(self.h, v)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        off = ptr - self.arena.data_ptr()
        assert off >= 0 and base <= ptr
        return self.arena[off:off + n * 4].view(torch.float32).clone()

    def params_tensor(self, v):
        """Device tensor copy (storage dtype) of local virtual stage v's flat parameter buffer."""
        ptr, n = B.jpp_stage_params(self.h, v)
        esz = 2 if self.w.dtype == inp.DT_BF16 else 4
        off = ptr - self.arena.data_ptr()
        return self.arena[off:off + n * esz].view(torch_dtype(self.w)).clone()

    def optimizer_bind(self, kind):
        """Allocates and binds the optimizer state (AdamW: fp32 master weights and moments)."""
        nbytes = B.jpp_stage_optimizer_bytes(self.h, kind)
        self.opt_state = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=self.dev)
        B.jpp_stage_optimizer_bind(self.h, kind, self.opt_state.data_ptr(), nbytes, self.compute.cuda_stream)

    def apply_gradients(self, kind, lr, **kw):
        B.jpp_stage_apply_gradients(self.h, kind, lr, self.compute.cuda_stream, **kw)

    def losses(self):
        ptr = B.jpp_stage_losses(self.h)
        off = ptr - self.arena.data_ptr()
        return self.arena[off:off + self.V * self.M * 4].view(torch.float32).clone().cpu().numpy().astype(np.float64)

    def results(self):
        """Everything the stage produced, as host float64 arrays keyed like the oracle's output."""
        self.sync()
        w, M = self.w, self.M
        out = {"y": {}, "dx": {}, "grads": {}, "loss": {}}
        for v, s in enumerate(w.stage_ids):
            if not w.loss_head:
                out["y"][s] = [to_host(self.out_y[v * M + i]) for i in range(M)]
            out["dx"][s] = [to_host(self.out_dx[v * M + i]) for i in range(M)]
            out["grads"][s] = self.unpack_grads(self.grads_tensor(v).cpu().numpy().astype(np.float64))
        if w.loss_head:
            l = self.losses()
            for v, s in enumerate(w.stage_ids):
                out["loss"][s] = list(l[v * M:(v + 1) * M])
        return out


def default_tasks(w):
    return B.jpp_schedule_make(w.sched, w.P, w.rank, w.V, w.n_microbatches)


class Pipeline:
    """P actors (Stage objects) of one pipeline on one device plus the pipeline's own boundary
    buffers and outer inputs / outputs.  `w` describes one actor (P, V, layer shape);
    w.loss_head says whether the last global stage ends in the loss."""

    def __init__(self, w, task_lists, dev="cuda:0"):
        from dataclasses import replace
        self.w, self.dev = w, dev
        self.P, self.V, self.M = w.P, w.V, w.n_microbatches
        self.S = self.P * self.V
        self.task_lists = [list(t) for t in task_lists]
        self.actors = [Stage(replace(w, rank=r, loss_head=(w.loss_head if r == self.P - 1 else 0),
                                     embed=(w.embed if r == 0 else 0)),
                             tasks=self.task_lists[r], dev=dev) for r in range(self.P)]
        nbytes = B.jpp_pipeline_arena_bytes(self.actors[0].cfg, self.P, self.M)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.h = B.jpp_pipeline_create([a.h for a in self.actors], base, nbytes)

    def close(self):
        if self.h is not None:
            B.jpp_pipeline_destroy(self.h)
            self.h = None
        for a in self.actors:
            a.close()

    def set_params_host(self, params_by_stage):
        for a in self.actors:
            a.set_params_host(params_by_stage)

    def set_params_random(self, seed=0):
        for r, a in enumerate(self.actors):
            a.set_params_random(seed=seed + r)

    def bind_random(self, seed=1):
        """Synthetic outer inputs generated in HBM (benchmark path)."""
        w, dt = self.w, torch_dtype(self.w)
        shp = (w.microbatch, w.seq_len, w.d_model)
        g = torch.Generator(device=self.dev)
        g.manual_seed(seed)
        if w.embed:
            self.x_in = [torch.randint(0, w.vocab, (w.microbatch, w.seq_len), generator=g, device=self.dev,
                                       dtype=torch.int32) for _ in range(self.M)]
        else:
            self.x_in = [torch.randn(shp, generator=g, device=self.dev).to(dt) for _ in range(self.M)]
        self.dx_out = [torch.zeros(shp, dtype=dt, device=self.dev) for _ in range(self.M)]
        self.tg = self.cot_in = self.y_out = None
        if w.loss_head:
            self.tg = [torch.randint(0, w.vocab, (w.microbatch, w.seq_len), generator=g, device=self.dev,
                                     dtype=torch.int32) for _ in range(self.M)]
        else:
            self.cot_in = [(torch.randn(shp, generator=g, device=self.dev) * w.cot_std).to(dt) for _ in range(self.M)]
            self.y_out = [torch.zeros(shp, dtype=dt, device=self.dev) for _ in range(self.M)]
        torch.cuda.synchronize()
        ptrs = lambda ts: [t.data_ptr() for t in ts] if ts else None
        B.jpp_pipeline_bind(self.h, ptrs(self.x_in), ptrs(self.dx_out), ptrs(self.tg), ptrs(self.cot_in),
                            ptrs(self.y_out))

    def bind(self, x0, cot_last=None, targets=None):
        w, dt = self.w, torch_dtype(self.w)
        shp = (w.microbatch, w.seq_len, w.d_model)
        if w.embed:      # x0: int32 token ids
            self.x_in = [torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.dev) for x in x0]
        else:
            self.x_in = [to_device(x, w, self.dev) for x in x0]
        self.dx_out = [torch.zeros(shp, dtype=dt, device=self.dev) for _ in range(self.M)]
        self.tg = self.cot_in = self.y_out = None
        if w.loss_head:
            self.tg = [torch.from_numpy(np.ascontiguousarray(t, dtype=np.int32)).to(self.dev) for t in targets]
        else:
            self.cot_in = [to_device(c, w, self.dev) for c in cot_last]
            self.y_out = [torch.zeros(shp, dtype=dt, device=self.dev) for _ in range(self.M)]
        torch.cuda.synchronize()
        ptrs = lambda ts: [t.data_ptr() for t in ts] if ts else None
        B.jpp_pipeline_bind(self.h, ptrs(self.x_in), ptrs(self.dx_out), ptrs(self.tg), ptrs(self.cot_in),
                            ptrs(self.y_out))

    def zero_grads(self):
        for a in self.actors:
            a.zero_grads()

    def run(self, task_lists=None):
        B.jpp_pipeline_run(self.h, self.task_lists if task_lists is None else task_lists,
                           [a.compute.cuda_stream for a in self.actors], [a.side.cuda_stream for a in self.actors])

    def sync(self):
        B.jpp_pipeline_sync(self.h)

    def sum_tied_gradients(self):
        """The one addition after the loop for a tied embedding / LM head (on actor 0's compute stream)."""
        B.jpp_pipeline_sum_tied_gradients(self.h, self.actors[0].compute.cuda_stream)

    def results(self):
        """Host float64 results keyed like oracle.pipeline_oracle.run_pipeline's output."""
        self.sync()
        torch.cuda.synchronize()
        out = {"grads": {}, "dx": [to_host(t) for t in self.dx_out]}
        for r, a in enumerate(self.actors):
            for v in range(self.V):
                g = a.unpack_grads(a.grads_tensor(v).cpu().numpy().astype(np.float64))
                if "head" in g and not (r == self.P - 1 and v == self.V - 1):
                    del g["head"]
                if "embed" in g and not (r == 0 and v == 0):
                    del g["embed"]
                out["grads"][v * self.P + r] = g
        if self.w.loss_head:
            l = self.actors[-1].losses()
            out["loss"] = list(l[(self.V - 1) * self.M:self.V * self.M])
        else:
            out["y"] = [to_host(t) for t in self.y_out]
        return out
