#!/usr/bin/env python3
"""Throughput of the data-parallel hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: index gather + scatter over workers -> sliced gradient
function -> worker reduce fused with the momentum update (config 2, the
default, and config 1); or the single stage a configuration isolates (3: reduce
+ update of ResNet-50-sized gradients, 4: normalising image gather, 5:
six-output sliced evaluation).  Prints ONE JSON line.

`roofline` is for the dominant kernel of the step: algorithmic bytes per launch
divided by that kernel's mean duration, measured here with events attached to
its launches inside the timed region.  With --graph the K timed steps are
replays of a HIP graph that holds the steps' launches (the calls of the library
only launch kernels, so a caller can capture them; launch gaps shrink), and the
dominant kernel is timed in a short eager pass before the timed region.
`cpu_baseline` is the NumPy float64 oracle timed on this machine's host cores on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published

# HBM bytes per launch of each config's dominant kernel, from rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE runs of this file (10 steps), scaled by what the same counters read for the
# plain copy of --config 0 (fetch x2.000, write x1.000).  Summaries: profiles/*_kernel_stats.txt.
MEASURED_TRAFFIC_BYTES = {2: 210.37e6, 3: 1226.75e6, 4: 192.83e6, 5: 264.56e6, 6: 59.08e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=2, choices=[0, 1, 2, 3, 4, 5, 6],
                    help="0 = plain copy of known size (calibrates the rocprofv3 byte counters)")
    ap.add_argument("--rule", default="momentum", choices=["momentum", "nesterov", "rmsprop", "adam"],
                    help="config 3 only: the update rule fused with the N-way average (Sec. 3.3)")
    ap.add_argument("--collective", default=None, choices=["all_reduce", "broadcast", "all_gather"],
                    help="config 3 shape only: time one collective over the 8 worker copies instead (Sec. 3.2)")
    ap.add_argument("--indexing", default="list", choices=["list", "slice", "resident"],
                    help="config 4 only: index list (default), slice-form indexes, or per-worker lists over "
                         "shares resident on the workers (Sec. 5.2)")
    ap.add_argument("--batch", type=int, default=None,
                    help="configs 1 and 2 only: minibatch size, to time worker shares that do not divide evenly "
                         "(default: the configuration's own, 256 / 1024)")
    ap.add_argument("--rows-per-worker", type=int, default=None,
                    help="config 2 only, a labelled supplementary shape (not the configuration): the same model and "
                         "kernels with this many rows per worker (e.g. 8192), to show what the products reach when "
                         "the per-worker shape does not bound them")
    ap.add_argument("--conv-shape", default=None,
                    help="config 6 at another block shape: H,W,C_in,C_out (e.g. 14,14,256,256)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the steps (one per rotating input set) into one HIP graph and time its replays; "
                         "the dominant kernel is then timed in a short eager pass before the timed region")
    ap.add_argument("--beside", default="valu:0",
                    help="--probe beside only: kind:count of the other instructions after each MFMA, valu:0|1|2|4|6|8|12 "
                         "or lds:1|2|4")
    ap.add_argument("--probe", default=None, choices=["mfma", "fill", "fetch", "read", "beside"],
                    help="config 0 only: instead of the copy, one of the library's peak probes (register-resident bf16 "
                         "MFMA loop; plain 16-byte stores over 1 GiB; operand tiles from L2 straight into LDS)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="the K timed steps are run this many times; value and ms_per_step are the median repeat's")
    ap.add_argument("--separate-gather", action="store_true",
                    help="configs 1, 2 and 6: input indexing as a gather call of its own before the sliced call "
                         "(default: folded into the sliced call)")
    ap.add_argument("--min-warmup-ms", type=float, default=60.0,
                    help="keep running untimed steps after the --warmup steps until this much time has passed "
                         "(0: exactly --warmup steps)")
    ap.add_argument("--sample-every", type=int, default=None,
                    help="put the per-kernel event pair on every N-th step only (default 8; 1 below 64 timed steps in all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def share_bounds(synk, count, parts):
    """[(start, stop)] of each worker's share, by the library's own split rule (Sec. 3.2 step 1)."""
    off = synk.synk_split(count, parts)
    return list(zip(off[:-1], off[1:]))


def share_sizes(synk, count, parts):
    return [b - a for a, b in share_bounds(synk, count, parts)]


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        n = [i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return 1


class Timer:
    """HIP events attached to launches inside the timed region: the library puts the pair on the selected
    kernel's own dispatch (begin and end timestamps of that kernel on the launch stream).  A step arms at
    most one pair, for one named target; targets rotate over the sampled steps.  Only every `every`-th
    step is sampled: a dispatch that carries events costs about 4 us more than one that does not (measured:
    config 5 at 53.4 us a call with a pair on every call, 49.4 without any), and that cost belongs to the
    measurement, not to the step."""

    def __init__(self, torch, synk, n, every=1):
        # events are created before the timed region: creating one costs more than a launch
        # (torch creates the underlying event at the first record)
        self.synk = synk
        self.pool = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                     for _ in range(n)]
        for a, b in self.pool:
            a.record()
            b.record()
        torch.cuda.synchronize()
        self.used, self.on, self.samples, self.every = 0, False, {}, max(1, every)

    def due(self, i):
        """True when step i is one of the sampled steps."""
        return self.on and i % self.every == 0

    def bracket(self, fn, name="dominant", kernel=0):
        """Runs fn(); with the timer on, the launch of `kernel` inside it carries the next event pair."""
        if self.used < len(self.pool):
            a, b = self.pool[self.used]
            self.used += 1
            self.synk.synk_profile_next_launch_of(kernel, a, b)
            fn()
            if self.synk.synk_profile_pending():      # the call did not launch that kernel: no sample
                self.synk.synk_profile_next_launch_of(kernel, None, None)
            else:
                self.samples.setdefault(name, []).append((a, b))
            return
        fn()

    def mean_ms(self, name="dominant"):
        ev = self.samples.get(name, [])
        return sum(a.elapsed_time(b) for a, b in ev) / max(len(ev), 1)

    def count(self, name="dominant"):
        return len(self.samples.get(name, []))


# ------------------------------------------------------------------ workloads
class MlpStep:
    """Configs 1 and 2: the whole synchronous-SGD step."""

    def __init__(self, torch, synk, cfg_no, batch=None, rows_per_worker=None, separate_gather=False):
        import numpy as np
        import workloads
        self.torch, self.s, self.np = torch, synk, np
        if cfg_no == 1:
            c = workloads.config1()
            c["idx_sets"] = [np.random.default_rng(i).permutation(4096)[:256].astype(np.int32) for i in range(8)]
        else:
            c = workloads.config2(n_index_sets=8)
        if rows_per_worker is not None:
            rng = np.random.default_rng(workloads.SEED_BASE + 2000)
            c["idx_sets"] = [rng.integers(0, c["data"].shape[0], c["n_workers"] * rows_per_worker).astype(np.int32)
                             for _ in range(2)]
        if batch is not None:
            if not 1 <= batch <= len(c["idx_sets"][0]):
                raise SystemExit("--batch must be in [1, %d] for this configuration" % len(c["idx_sets"][0]))
            c["idx_sets"] = [ix[:batch] for ix in c["idx_sets"]]
        self.c = c
        self.dims, self.N, self.S = c["dims"], c["n_workers"], c["n_slices"]
        self.bf16 = c["compute"] == "bf16"
        self.cd = synk.SYNK_BF16 if self.bf16 else synk.SYNK_F32
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.data, self.labels = up(c["data"]), up(c["labels"])
        self.idx = [up(i) for i in c["idx_sets"]]
        self.B = len(c["idx_sets"][0])
        self.P = synk.synk_mlp_param_count(self.dims)
        self.p, self.v = up(c["theta"]), torch.zeros(self.P, device="cuda")
        self.p_lp = torch.zeros(self.P, dtype=torch.bfloat16, device="cuda") if self.bf16 else None
        if self.bf16:
            synk.synk_cast_bf16(self.p, self.p_lp)
        self.rows = share_sizes(synk, self.B, self.N)
        xdt = torch.bfloat16 if self.bf16 else torch.float32
        self.x = [torch.zeros((n, self.dims[0]), dtype=xdt, device="cuda") for n in self.rows]
        self.y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in self.rows]
        self.grad = [torch.zeros(self.P, device="cuda") for _ in self.rows]
        self.loss = torch.zeros(self.N, device="cuda")
        self.loss_out = torch.zeros(1, device="cuda")
        self.ws = torch.empty(synk.synk_sliced_grad_workspace_bytes(self.dims, self.cd, self.rows),
                              dtype=torch.uint8, device="cuda")
        self.units, self.unit = self.B, "samples/s"
        self.dtype = "bf16" if self.bf16 else "f32"
        self.workload = ("config 2: wide MLP 3072-1024-1024-10 step, batch %d, 8 worker shares x 4 slices, "
                         "bf16 GEMM inputs / fp32 accumulate" % self.B if cfg_no == 2 else
                         "config 1: tiny MLP 784-256-10 step, batch %d, 2 worker shares x 4 slices, fp32" % self.B)
        if batch is not None:
            self.workload += " (worker shares %s)" % "/".join(str(r) for r in sorted(set(self.rows), reverse=True))
        if rows_per_worker is not None:
            self.workload = ("SUPPLEMENTARY shape, not a configuration: the config-2 model and kernels at %d rows per "
                             "worker (batch %d)" % (rows_per_worker, self.B))
        # dominant kernel: the fused N-way reduce + momentum update.  Per parameter it reads N
        # gradients, reads and writes p and v (fp32) and, with bf16 compute, writes the bf16 copy.
        self.dom_name = "reduce_sgd_kernel"
        self.dom_bytes = self.P * (4 * self.N + 16 + (2 if self.bf16 else 0))
        # Input indexing: folded into the sliced call (the first product reads its rows through the index;
        # the dataset is resident in the compute type), or with --separate-gather as a call of its own
        # that converts from the fp32 dataset.
        self.indexed = not separate_gather
        self.workload += ("; input indexing inside the sliced call (dataset resident in %s)" % self.dtype
                          if self.indexed else "; input indexing as a gather call of its own")
        self.targets, self.kernel_work = self._plan(synk)

        # the C calls of a step, arguments marshalled once (launch cost, not Python cost, per step)
        s = synk
        if self.indexed:
            self.data_c = self.data
            if self.bf16:
                self.data_c = torch.empty(self.data.shape, dtype=torch.bfloat16, device="cuda")
                s.synk_cast_bf16(self.data, self.data_c)
            self.ws = torch.empty(s.synk_sliced_grad_indexed_workspace_bytes(self.dims, self.cd, self.B, self.N),
                                  dtype=torch.uint8, device="cuda")
            self.call_gather = [None] * len(self.idx)
            self.call_grads = [s.prepare(s.synk_sliced_grad_indexed, self.dims, self.cd, self.p, self.p_lp, self.data_c,
                                         self.labels, ix, self.S, s.SYNK_MEAN, self.grad, self.loss, self.ws)
                               for ix in self.idx]
        else:
            self.call_gather = [s.prepare(s.synk_gather_rows, self.data, ix, self.x, labels=self.labels,
                                          dst_labels=self.y) for ix in self.idx]
            self.call_grads = [s.prepare(s.synk_sliced_grad, self.dims, self.cd, self.p, self.p_lp, self.x, self.y,
                                         self.rows, self.S, s.SYNK_MEAN, self.grad, self.loss, self.ws)] * len(self.idx)
        self.call_update = s.prepare(s.synk_reduce_sgd_update, self.grad, self.p, self.v, c["lr"], c["momentum"],
                                     c["weight_decay"], p_lp=self.p_lp, loss_in=self.loss, loss_out=self.loss_out)

    cycle = 8          # distinct steps (rotating index sets)

    def _plan(self, s):
        """Which launches a step makes and what each does: (name, call, kernel id) per target, and per name
        the algorithmic flops and bytes of one launch (stated in the design notes).  The launch plan is the
        library's for these two configurations' shapes."""
        d, B, N, e = self.dims, self.B, self.N, (2 if self.bf16 else 4)
        L = len(d) - 1
        dW = lambda l: dict(flops=2.0 * B * d[l - 1] * d[l],
                            bytes=N * (d[l - 1] * d[l] + d[l]) * 4 + B * (d[l - 1] + d[l]) * e,
                            write_bytes=N * (d[l - 1] * d[l] + d[l]) * 4)
        fwd = lambda l: dict(flops=2.0 * B * d[l - 1] * d[l], bytes=(B * d[l - 1] + d[l - 1] * d[l] + B * d[l]) * e)
        work = {"gather": dict(bytes=B * (d[0] * 4 + d[0] * e + 8)),
                "reduce_update": dict(bytes=self.dom_bytes)}
        targets = [("forward_1", "grad", s.SYNK_KERNEL_MAIN)]
        work["forward_1"] = fwd(1)
        if not self.indexed:
            targets.insert(0, ("gather", "gather", s.SYNK_KERNEL_MAIN))
        else:
            work["forward_1"]["bytes"] += B * (d[0] * e + 8)       # it also leaves the rows and labels behind
        for l in range(2, L):
            targets.append(("forward_%d" % l, "grad", s.SYNK_KERNEL_MLP_FORWARD(l)))
            work["forward_%d" % l] = fwd(l)
        # last layer: logits, softmax cross-entropy, dZ_L and dZ_{L-1} in one launch
        targets.append(("head", "grad", s.SYNK_KERNEL_MLP_HEAD))
        work["head"] = dict(flops=4.0 * B * d[L - 1] * d[L], bytes=B * d[L - 1] * e * 2 + d[L - 1] * d[L] * e)
        if L >= 3:
            # dW_L, dW_{L-1} and dZ_{L-2} share one launch
            targets.append(("backward_group", "grad", s.SYNK_KERNEL_MLP_BACKWARD_GROUP))
            g = dict(flops=dW(L)["flops"] + dW(L - 1)["flops"] + 2.0 * B * d[L - 2] * d[L - 1],
                     bytes=dW(L)["bytes"] + dW(L - 1)["bytes"] + (B * d[L - 1] + d[L - 2] * d[L - 1] + 2 * B * d[L - 2]) * e,
                     write_bytes=dW(L)["write_bytes"] + dW(L - 1)["write_bytes"] + B * d[L - 2] * e)
            work["backward_group"] = g
            rest = range(L - 2, 0, -1)
        elif L == 2:
            # dW_2 and dW_1 share one launch when the shapes allow it, else they are launched one by one:
            # targets for both forms; the form that does not occur yields no samples
            targets.append(("backward_group", "grad", s.SYNK_KERNEL_MLP_BACKWARD_GROUP))
            work["backward_group"] = dict(flops=dW(2)["flops"] + dW(1)["flops"], bytes=dW(2)["bytes"] + dW(1)["bytes"],
                                          write_bytes=dW(2)["write_bytes"] + dW(1)["write_bytes"])
            rest = range(L, 0, -1)
        else:
            rest = range(L, 0, -1)
        for l in rest:
            targets.append(("dw_%d" % l, "grad", s.SYNK_KERNEL_MLP_DW(l)))
            work["dw_%d" % l] = dW(l)
        targets.append(("reduce_update", "update", s.SYNK_KERNEL_MAIN))
        return targets, work

    def step(self, i, timer):
        gather = self.call_gather[i % len(self.call_gather)]
        call_grad = self.call_grads[i % len(self.call_grads)]
        if not timer.due(i):
            if gather:
                gather()
            call_grad()
            self.call_update()
            return
        name, call, kernel = self.targets[(i // timer.every) % len(self.targets)]
        if call == "gather":
            timer.bracket(gather, name, kernel)
        elif gather:
            gather()
        if call == "grad":
            timer.bracket(call_grad, name, kernel)
        else:
            call_grad()
        if call == "update":
            timer.bracket(self.call_update, name, kernel)
        else:
            self.call_update()

    def kernel_report(self, timer):
        """Per-launch figures of every kernel of the step, from the events attached to its dispatches."""
        peak_mfma = 2500.0 if self.bf16 else 157.3
        out = []
        for name, _, _ in self.targets:
            ms, wk = timer.mean_ms(name), self.kernel_work[name]
            if timer.count(name) == 0 or ms <= 0:
                continue
            r = {"kernel": name, "us": ms * 1e3, "samples": timer.count(name)}
            if "flops" in wk:
                tf = wk["flops"] / (ms * 1e-3) / 1e12
                r.update(flops=wk["flops"], tflops=tf, frac_mfma=tf / peak_mfma, mfma_peak_tflops=peak_mfma)
            gbs = wk["bytes"] / (ms * 1e-3) / 1e9
            r.update(bytes=wk["bytes"], gbs=gbs, frac_hbm=gbs / HBM_PEAK_GBS)
            if "write_bytes" in wk:
                r["write_gbs"] = wk["write_bytes"] / (ms * 1e-3) / 1e9
            out.append(r)
        return out

    def cpu_baseline(self):
        from oracle import mlp as omlp, update as oupdate
        c, np = self.c, self.np
        theta, v = c["theta"].astype(np.float64), np.zeros(self.P)
        best = 1e30
        for rep in range(3):
            t0 = time.perf_counter()
            loss, g = omlp.full(theta, self.dims, c["data"], c["labels"], c["idx_sets"][rep % len(c["idx_sets"])])
            oupdate.sgd_momentum(theta, v, g, c["lr"], c["momentum"], c["weight_decay"])
            best = min(best, time.perf_counter() - t0)
        return self.B / best, "3 whole steps (full-batch oracle: gather, fwd/bwd, update), best of 3"


class ReduceStep:
    """Config 3: N-way average of ResNet-50-sized gradients fused with the update rule."""

    HYPER = dict(nesterov=dict(lr=0.1, momentum=0.9, weight_decay=1e-4),
                 rmsprop=dict(lr=0.01, rho=0.9, eps=1e-6, weight_decay=1e-4),
                 adam=dict(lr=0.001, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-4))

    def __init__(self, torch, synk, rule="momentum"):
        import numpy as np
        import workloads
        self.torch, self.s, self.np = torch, synk, np
        c = workloads.config3()
        self.c, self.rule = c, rule
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.P, self.N = c["n_params"], c["n_workers"]
        # 3 rotating gradient sets (2.4 GB) so that the 256 MB last-level cache cannot serve the reads
        self.grads = [[up(g) for g in c["grads"]]]
        for k in range(2):
            self.grads.append([g.roll(k + 1) for g in self.grads[0]])
        self.p, self.v = up(c["p"]), up(c["v"])
        self.loss_in, self.loss_out = up(c["losses"]), torch.zeros(1, device="cuda")
        self.units, self.unit = self.P, "params/s"
        self.dtype = "f32"
        n_state = 2 if rule == "adam" else 1
        self.dom_bytes = self.P * (4 * self.N + 8 + 8 * n_state)
        if rule == "momentum":
            self.workload = ("config 3: average of 8 ResNet-50-sized fp32 gradient buffers (25,557,032 params, 161 "
                             "tensors) fused with momentum SGD (lr .1, m .9, wd 1e-4) and the scalar-loss mean")
            self.dom_name = "reduce_sgd_kernel"
            self.calls = [synk.prepare(synk.synk_reduce_sgd_update, gs, self.p, self.v, c["lr"], c["momentum"],
                                       c["weight_decay"], loss_in=self.loss_in, loss_out=self.loss_out)
                          for gs in self.grads]
        else:
            h = self.HYPER[rule]
            self.workload = ("config 3 shape with the %s rule: average of 8 ResNet-50-sized fp32 gradient buffers "
                             "(25,557,032 params) fused with the update (%s) and the scalar-loss mean" %
                             (rule, ", ".join("%s %g" % kv for kv in h.items())))
            self.dom_name = "reduce_update_kernel"
            self.s2 = torch.zeros_like(self.v) if rule == "adam" else None
            # the step number only enters the host-side bias correction of Adam; a fixed one times the same work
            self.calls = [synk.prepare(synk.synk_reduce_update, rule, gs, self.p, self.v, self.s2, step=1000,
                                       loss_in=self.loss_in, loss_out=self.loss_out, **h)
                          for gs in self.grads]

    cycle = 3

    def step(self, i, timer):
        if timer.due(i):
            timer.bracket(self.calls[i % 3])
        else:
            self.calls[i % 3]()

    def cpu_baseline(self):
        from oracle import reduce as oreduce, update as oupdate
        c = self.c
        best = 1e30
        for _ in range(3):
            t0 = time.perf_counter()
            if self.rule == "momentum":
                oupdate.reduce_and_update(c["p"], c["v"], c["grads"], c["lr"], c["momentum"], c["weight_decay"],
                                          None, c["losses"])
            else:
                G = oreduce.reduce_buffers(list(c["grads"]), "mean")
                oupdate.apply_rule(self.rule, c["p"], c["v"], c["v"], G, dict(self.HYPER[self.rule], t=1000))
            best = min(best, time.perf_counter() - t0)
        return self.P / best, "3 whole steps at full size, best of 3"


class CollectiveStep:
    """Config 3's shape (8 worker copies of a 25,557,032-element fp32 array) under one collective of Sec. 3.2."""

    def __init__(self, torch, synk, which):
        import numpy as np
        import workloads
        self.torch, self.s, self.np, self.which = torch, synk, np, which
        c = workloads.config3()
        self.c = c
        self.P, self.N = c["n_params"], c["n_workers"]
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.bufs = [up(g) for g in c["grads"]]
        self.units, self.unit, self.dtype = self.P, "params/s", "f32"
        if which == "all_reduce":
            # in place on 818 MB of buffers: values decay towards the mean, the traffic stays the same
            self.call = synk.prepare(synk.synk_all_reduce, self.bufs, "mean")
            self.dom_name, self.dom_bytes = "all_reduce_kernel", self.P * 4 * 2 * self.N
            what = "all-reduce (mean: the parameter / gradient average), in place"
        elif which == "broadcast":
            self.src = up(c["p"])
            self.call = synk.prepare(synk.synk_broadcast, self.src, self.bufs)
            self.dom_name, self.dom_bytes = "broadcast_kernel", self.P * 4 * (1 + self.N)
            what = "broadcast of one array to the 8 copies"
        else:
            self.bounds = share_bounds(synk, self.P, self.N)
            self.srcs = [up(c["p"][a:b]) for a, b in self.bounds]
            self.call = synk.prepare(synk.synk_all_gather, self.srcs, self.bufs)
            self.dom_name, self.dom_bytes = "all_gather_kernel", self.P * 4 * (1 + self.N)
            what = "all-gather of 8 equal shares into the 8 copies"
        self.workload = "config 3 shape (8 x 25,557,032 fp32): " + what

    def step(self, i, timer):
        if timer.due(i):
            timer.bracket(self.call)
        else:
            self.call()

    def cpu_baseline(self):
        from oracle import collectives as ocoll
        c = self.c
        best = 1e30
        for _ in range(3):
            t0 = time.perf_counter()
            if self.which == "all_reduce":
                ocoll.all_reduce(list(c["grads"]), "mean")
            elif self.which == "broadcast":
                ocoll.broadcast(c["p"], self.N)
            else:
                ocoll.all_gather([c["p"][a:b] for a, b in self.bounds])
            best = min(best, time.perf_counter() - t0)
        return self.P / best, "3 whole calls at full size, best of 3"


class GatherStep:
    """Config 4: uint8 image gather + per-channel normalise to fp32, 8 worker shares."""

    def __init__(self, torch, synk, indexing="list"):
        import numpy as np
        import workloads
        self.torch, self.s, self.np, self.indexing = torch, synk, np, indexing
        small = workloads.config4(n_data=8, batch=8)             # mean/std recipe
        self.mean, self.std = small["mean"], small["std"]
        self.n_data, self.B, self.N, self.chw = 50000, 256, 8, (3, 224, 224)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(workloads.SEED_BASE + 4)
        row = 3 * 224 * 224
        self.data = torch.empty((self.n_data, row), dtype=torch.uint8, device="cuda")
        for a in range(0, self.n_data, 5000):                    # 7.5 GB, filled on the device in pieces
            self.data[a:a + 5000] = torch.randint(0, 256, (5000, row), dtype=torch.uint8, device="cuda",
                                                  generator=gen)
        rng = workloads.rng_for(4, salt=1)
        self.labels = torch.from_numpy(rng.integers(0, 1000, self.n_data).astype(np.int32)).cuda()
        self.idx = [torch.from_numpy(rng.integers(0, self.n_data, self.B).astype(np.int32)).cuda()
                    for _ in range(64)]                          # fresh indexes every step
        self.lut = torch.empty(3 * 256, device="cuda")
        synk.synk_build_norm_lut(self.mean, self.std, self.lut)
        rows = share_sizes(synk, self.B, self.N)
        self.dst = [torch.zeros((n, row), device="cuda") for n in rows]
        self.dl = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in rows]
        self.units, self.unit = self.B, "images/s"
        self.dtype = "u8"
        self.workload = ("config 4: gather 256 of 50000 uint8 3x224x224 images by random index, normalise to "
                         "fp32 NCHW, 8 worker shares of 32, with labels")
        self.dom_name = "gather_u8_lut_kernel"
        self.dom_bytes = self.B * (row + 4 * row + 8)

        if indexing == "list":
            self.calls = [synk.prepare(synk.synk_gather_rows, self.data, ix, self.dst, lut=self.lut, channels=3,
                                       labels=self.labels, dst_labels=self.dl) for ix in self.idx]
        elif indexing == "slice":
            # 256 rows start, start+190, ...: a different start every step
            self.workload = ("config 4 shape with slice-form indexes: rows start::190 (256 of 50000 uint8 3x224x224 "
                             "images), normalise to fp32, 8 worker shares of 32, with labels")
            self.calls = [synk.prepare(synk.synk_gather_slice, self.data, s0, s0 + 256 * 190, 190, self.dst,
                                       lut=self.lut, channels=3, labels=self.labels, dst_labels=self.dl)
                          for s0 in [(k * 37) % 1000 for k in range(64)]]
        else:
            # the dataset scattered by first dimension into 8 resident shares of 6250 images (views of one
            # allocation); every worker excerpts 32 rows of its own share with its own list
            self.workload = ("config 4 shape with resident shares: 8 workers x 32 own indexes into their 6250-image "
                             "uint8 share, normalise to fp32, with labels")
            bounds = share_bounds(synk, self.n_data, self.N)
            shares = [self.data[a:b] for a, b in bounds]
            lshares = [self.labels[a:b] for a, b in bounds]
            self.lists = [[torch.from_numpy(rng.integers(0, b - a, n).astype(np.int32)).cuda()
                           for (a, b), n in zip(bounds, rows)] for _ in range(64)]
            self.calls = [synk.prepare(synk.synk_gather_resident, shares, ls, self.dst, lut=self.lut, channels=3,
                                       labels=lshares, dst_labels=self.dl) for ls in self.lists]

    cycle = 64

    def step(self, i, timer):
        if timer.due(i):
            timer.bracket(self.calls[i % 64])
        else:
            self.calls[i % 64]()

    def cpu_baseline(self):
        from oracle import gather as og
        np = self.np
        rng = np.random.default_rng(0)
        data = rng.integers(0, 256, (512,) + self.chw, dtype=np.uint8)     # 77 MB stand-in dataset
        idx = rng.integers(0, 512, self.B)
        best = 1e30
        for _ in range(3):
            t0 = time.perf_counter()
            for part in og.gather_shares(data, idx, self.N):
                og.normalise_u8(part, self.mean, self.std)
            best = min(best, time.perf_counter() - t0)
        return self.B / best, "3 whole batches of 256 from a 512-image host dataset, best of 3"


class EvalStep:
    """Config 5: six-output evaluation over 64 slices with aggregation."""

    def __init__(self, torch, synk):
        import numpy as np
        import workloads
        self.torch, self.s, self.np = torch, synk, np
        self.rows, self.C, self.S = 65536, 1000, 64
        self.host = workloads.config5()
        # 4 rotating input sets (1.05 GB) against the 256 MB last-level cache
        self.logits = [torch.from_numpy(self.host["logits"]).cuda()]
        for k in range(3):
            self.logits.append(self.logits[0].roll(k + 1, dims=0).contiguous())
        self.labels = torch.from_numpy(self.host["labels"]).cuda()
        z = lambda n, dt: torch.zeros(n, dtype=dt, device="cuda")
        self.out = (z(1, torch.float32), z(self.C, torch.int32), z(1, torch.float32), z(1, torch.float32),
                    z(1, torch.int32), z(self.rows, torch.int32))
        self.ws = torch.empty(synk.synk_sliced_eval_workspace_bytes(self.rows, self.C, self.S),
                              dtype=torch.uint8, device="cuda")
        self.units, self.unit = self.rows, "rows/s"
        self.dtype = "f32"
        self.workload = ("config 5: 65536 rows of 1000-class fp32 logits, 64 slices, outputs CE sum, class "
                         "counts, max, min, top-1 correct, argmax, aggregated over slices")
        # one call = two kernels (stage 1, stage 2); the event pair sits on stage 1's dispatch
        self.dom_name = "eval_stage1_regular_kernel"
        self.dom_bytes = self.rows * (4 * self.C + 8)
        self.calls = [synk.prepare(synk.synk_sliced_eval, lg, self.labels, self.S, *self.out, self.ws)
                      for lg in self.logits]

    cycle = 4

    def step(self, i, timer):
        if timer.due(i):
            timer.bracket(self.calls[i % 4])
        else:
            self.calls[i % 4]()

    def cpu_baseline(self):
        from oracle import evalops
        n = 4096
        t0 = time.perf_counter()
        evalops.sliced(self.host["logits"][:n], self.host["labels"][:n], 4)
        return n / (time.perf_counter() - t0), "4096 of the 65536 rows, 4 slices (the argmax loop is pure Python)"


class ConvStep:
    """Config 6: the whole step with the conv + batch-norm block as the function."""

    def __init__(self, torch, synk, conv_shape=None, separate_gather=False):
        import numpy as np
        import workloads
        self.torch, self.s, self.np = torch, synk, np
        if conv_shape:
            H, W, cin, cout = [int(v) for v in conv_shape.split(",")]
            c = self.c = workloads.config6(shape=(H, W, cin, cout, 1000))
        else:
            c = self.c = workloads.config6()
        rng = np.random.default_rng(6)
        idx_sets = [c["idx"]] + [rng.integers(0, c["data"].shape[0], len(c["idx"])).astype(np.int32) for _ in range(3)]
        self.shape, self.N, self.S = c["shape"], c["n_workers"], c["n_slices"]
        H, W, cin, cout, classes = self.shape
        self.bf16 = c["compute"] == "bf16"
        self.cd = synk.SYNK_BF16 if self.bf16 else synk.SYNK_F32
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.data, self.labels = up(c["data"]), up(c["labels"])
        self.B = len(c["idx"])
        self.P = synk.synk_convblock_param_count(self.shape)
        self.p, self.v = up(c["theta"]), torch.zeros(self.P, device="cuda")
        self.rows = share_sizes(synk, self.B, self.N)
        xdt = torch.bfloat16 if self.bf16 else torch.float32
        self.x = [torch.zeros((n, H * W * cin), dtype=xdt, device="cuda") for n in self.rows]
        self.y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in self.rows]
        self.grad = [torch.zeros(self.P, device="cuda") for _ in self.rows]
        self.loss = torch.zeros(self.N, device="cuda")
        self.loss_out = torch.zeros(1, device="cuda")
        self.ws = torch.empty(synk.synk_sliced_grad_conv_workspace_bytes(self.shape, self.cd, self.rows, self.S,
                                                                         c["eps"]), dtype=torch.uint8, device="cuda")
        self.units, self.unit = self.B, "samples/s"
        self.dtype = "bf16" if self.bf16 else "f32"
        self.workload = ("config 6: conv3x3 + batch-norm + ReLU block %dx%dx%d -> %d, pool, %d-way softmax; step "
                         "with batch %d over %d worker shares x %d slice, bf16 contraction inputs / fp32 "
                         "accumulate" % (H, W, cin, cout, classes, self.B, self.N, self.S))
        # dominant kernel: the forward convolution, a [pixels x 9 C_in] . [9 C_in x C_out] contraction (its
        # weight gradient has as many flops and takes about as long)
        held = self.bf16 and cin == 64 and cout <= 64 and W + 2 <= 63      # the shapes that kernel takes
        self.dom_name = "conv3x3_fwd_hold_kernel" if held else "conv3x3_fwd_patch_kernel"
        self.dom_bound, self.dom_unit = "mfma", "TFLOP/s"
        self.dom_peak = 2500.0 if self.bf16 else 157.3
        self.dom_work = 2.0 * self.B * H * W * 9 * cin * cout       # flops per launch
        self.dom_bytes = self.B * H * W * (cin + cout) * (2 if self.bf16 else 4)
        s = synk
        # Input indexing inside the sliced call (the convolution kernels read the images through the index
        # list; dataset resident in the compute type), or with --separate-gather as a call of its own.
        self.indexed = not separate_gather
        self.workload += ("; input indexing inside the sliced call (dataset resident in %s)" % self.dtype
                          if self.indexed else "; input indexing as a gather call of its own")
        if self.indexed:
            self.data_c = self.data
            if self.bf16:
                self.data_c = torch.empty(self.data.shape, dtype=torch.bfloat16, device="cuda")
                s.synk_cast_bf16(self.data, self.data_c)
            self.ws = torch.empty(s.synk_sliced_grad_conv_indexed_workspace_bytes(self.shape, self.cd, self.B, self.N,
                                                                                  self.S, c["eps"]),
                                  dtype=torch.uint8, device="cuda")
            self.call_gather = [None] * len(idx_sets)
            self.call_grads = [s.prepare(s.synk_sliced_grad_conv_indexed, self.shape, self.cd, c["eps"], self.p,
                                         self.data_c, self.labels, up(ix), self.S, s.SYNK_MEAN, self.grad, self.loss,
                                         self.ws) for ix in idx_sets]
        else:
            self.call_gather = [s.prepare(s.synk_gather_rows, self.data, up(ix), self.x, labels=self.labels,
                                          dst_labels=self.y) for ix in idx_sets]
            self.call_grads = [s.prepare(s.synk_sliced_grad_conv, self.shape, self.cd, c["eps"], self.p, self.x, self.y,
                                         self.rows, self.S, s.SYNK_MEAN, self.grad, self.loss, self.ws)] * len(idx_sets)
        self.call_update = s.prepare(s.synk_reduce_sgd_update, self.grad, self.p, self.v, c["lr"], c["momentum"],
                                     c["weight_decay"], loss_in=self.loss, loss_out=self.loss_out)

    cycle = 4

    def step(self, i, timer):
        k = i % len(self.call_gather)
        if self.call_gather[k]:
            self.call_gather[k]()
        if timer.due(i):
            timer.bracket(self.call_grads[k])
        else:
            self.call_grads[k]()
        self.call_update()

    def cpu_baseline(self):
        from oracle import convblock as oconv, gather as ogather, update as oupdate
        c, np = self.c, self.np
        theta, v = c["theta"].astype(np.float64), np.zeros(self.P)
        n = self.rows[0]
        t0 = time.perf_counter()
        for k in range(2):
            ix = c["idx"][k * n:(k + 1) * n]
            _, g = oconv.function(theta, self.shape, ogather.gather_rows(c["data"], ix),
                                  ogather.gather_rows(c["labels"], ix), c["eps"])
            oupdate.sgd_momentum(theta, v, g, c["lr"], c["momentum"], c["weight_decay"])
        return 2 * n / (time.perf_counter() - t0), "2 of the 8 worker shares (8 images each): function + update"


class ProbeStep:
    """Config 0 with --probe: a measured peak of the part (timing kernel of the library, nothing of the method)."""

    def __init__(self, torch, synk, which, beside="valu:0"):
        self.s, self.which = synk, which
        if which == "beside":
            kind, n = beside.split(":")
            pid = (synk.SYNK_PROBE_MFMA_BESIDE_VALU if kind == "valu" else synk.SYNK_PROBE_MFMA_BESIDE_LDS) + int(n)
            self.buf, self.iters = torch.zeros(64, device="cuda"), 20000
            self.unit, self.dom_bound, self.dom_unit, self.dom_peak = "flop/s", "mfma", "TFLOP/s", 2500.0
            self.workload = ("probe: 256 workgroups x 4 wavefronts (one per SIMD) x 40000 bf16 32x32x16 MFMAs, %s %s "
                             "after each" % (n, "vector-ALU additions" if kind == "valu" else "4-byte LDS reads"))
            self.mfmas_per_wave = 2 * self.iters
        elif which == "mfma":
            self.buf, self.iters, pid = torch.zeros(64, device="cuda"), 20000, synk.SYNK_PROBE_MFMA_BF16
            self.unit, self.dom_bound, self.dom_unit, self.dom_peak = "flop/s", "mfma", "TFLOP/s", 2500.0
            self.workload = "probe: 512 workgroups x 8 wavefronts x 20000 x 4 bf16 32x32x16 MFMAs on registers"
        elif which == "fill":
            self.buf, self.iters, pid = torch.empty(1 << 28, device="cuda"), 1, synk.SYNK_PROBE_FILL
            self.unit = "bytes/s"
            self.workload = "probe: 1 GiB of 16-byte stores, one per thread, in address order"
        elif which == "read":
            self.buf, self.iters, pid = torch.ones(1 << 28, device="cuda"), 1, synk.SYNK_PROBE_READ
            self.unit = "bytes/s"
            self.workload = "probe: 1 GiB of 16-byte loads, eight per thread, 32 KB a workgroup in address order"
        else:
            self.buf, self.iters, pid = torch.ones(2 << 20, device="cuda"), 48, synk.SYNK_PROBE_LDS_FETCH
            self.unit = "bytes/s"
            # nominal L1 fill rate: 64 B/clk per CU, 256 CUs, 2.4 GHz
            self.dom_bound, self.dom_unit, self.dom_peak = "l2", "GB/s", 64 * 256 * 2.4
            self.workload = ("probe: 256 workgroups each bringing 48 tiles of 128 rows x 128 B (pitch 6 KB) from L2 "
                             "straight into LDS")
        self.pid = pid
        self.units = synk.synk_probe_launch(pid, self.buf, self.iters)      # work of one launch
        self.dom_work, self.dom_bytes = self.units, self.units
        self.dtype = "bf16" if which in ("mfma", "beside") else "u8"
        self.dom_name = "probe_%s_kernel" % which

    def step(self, i, timer):
        fn = lambda: self.s.synk_probe_launch(self.pid, self.buf, self.iters)
        if timer.due(i):
            timer.bracket(fn)
        else:
            fn()

    def cpu_baseline(self):
        return 0.0, "none"


class CopyStep:
    """Config 0: a plain copy kernel of known size (1 GiB in, 1 GiB out), against which the
    FETCH_SIZE / WRITE_SIZE counters of the other kernels are scaled."""

    def __init__(self, torch, synk):
        n = 256 * 1024 * 1024
        self.src = [torch.full((n,), float(k + 1), device="cuda") for k in range(2)]
        self.dst = torch.empty(n, device="cuda")
        self.calls = [synk.prepare(synk.synk_reduce_buffers, [b], synk.SYNK_SUM, self.dst) for b in self.src]
        self.units, self.unit, self.dtype = n, "elements/s", "f32"
        self.workload = "config 0: copy of 2^28 fp32 (synk_reduce_buffers with one buffer)"
        self.dom_name, self.dom_bytes = "reduce_kernel", 8 * n

    cycle = 2

    def step(self, i, timer):
        if timer.due(i):
            timer.bracket(self.calls[i % 2])
        else:
            self.calls[i % 2]()

    def cpu_baseline(self):
        return 0.0, "none"


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    from paper_1710_04162_amd import binding as synk
    torch.cuda.set_device(0)

    if a.graph:
        # capture needs a stream of its own; the calls below are prepared on it
        torch.cuda.set_stream(torch.cuda.Stream())
    wl = {0: lambda: (ProbeStep(torch, synk, a.probe, a.beside) if a.probe else CopyStep(torch, synk)), 1: lambda: MlpStep(torch, synk, 1, a.batch, separate_gather=a.separate_gather), 2: lambda: MlpStep(torch, synk, 2, a.batch, a.rows_per_worker, a.separate_gather),
          3: lambda: (CollectiveStep(torch, synk, a.collective) if a.collective else ReduceStep(torch, synk, a.rule)), 4: lambda: GatherStep(torch, synk, a.indexing),
          5: lambda: EvalStep(torch, synk), 6: lambda: ConvStep(torch, synk, a.conv_shape, a.separate_gather)}[a.config]()
    steps = a.steps if a.steps is not None else {0: 50, 1: 5000, 2: 4500, 3: 2800, 4: 5000, 5: 5000, 6: 3200}[a.config]   # >= 0.5 s a repeat
    if a.rows_per_worker is not None and a.steps is None:
        steps = 56
    warmup = a.warmup if a.warmup is not None else 20

    repeats = max(1, a.repeats)
    per_repeat = []
    if a.graph:
        # dominant kernel: a short eager pass with the events on its dispatches
        probe = 56
        timer = Timer(torch, synk, probe)
        for i in range(warmup):
            wl.step(i, timer)
        torch.cuda.synchronize()
        timer.on = True
        for i in range(probe):
            wl.step(i, timer)
        torch.cuda.synchronize()
        timer.on = False
        # one graph holding `cycle` consecutive steps; K steps = K // cycle replays + the rest eagerly
        cycle = getattr(wl, "cycle", 1)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=torch.cuda.current_stream()):
            for i in range(cycle):
                wl.step(i, timer)
        for _ in range(max(1, warmup // cycle)):
            g.replay()
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps // cycle):
                g.replay()
            for i in range(steps % cycle):
                wl.step(i, timer)
            torch.cuda.synchronize()
            per_repeat.append(time.perf_counter() - t0)
    else:
        every = a.sample_every if a.sample_every else (8 if steps * repeats >= 64 else 1)
        timer = Timer(torch, synk, steps * repeats // every + repeats + 1, every)
        for i in range(warmup):
            wl.step(i, timer)
        torch.cuda.synchronize()
        # The part needs about 25 ms of work to reach its steady clocks (20-step repeats after 5 warm-up
        # steps read 112.9, 111.0, 109.4 ... 105 us a step over the first ten): with a short warm-up count
        # the untimed steps go on, in batches of 20, until 60 ms have passed.
        warm_t0, warm_more = time.perf_counter(), 0
        while a.min_warmup_ms > 0 and (time.perf_counter() - warm_t0) * 1e3 < a.min_warmup_ms:
            for i in range(20):
                wl.step(warmup + warm_more + i, timer)
            torch.cuda.synchronize()
            warm_more += 20
        timer.on = True
        for r in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(r * steps, (r + 1) * steps):
                wl.step(i, timer)
            torch.cuda.synchronize()
            per_repeat.append(time.perf_counter() - t0)
    dt = sorted(per_repeat)[len(per_repeat) // 2]          # the median repeat of exactly K steps

    # The event pair sits on the kernel's own dispatch: begin-to-end time of the kernel, the same
    # quantity as the kernel duration in a rocprofv3 kernel trace.
    dom_ms = timer.mean_ms("reduce_update" if hasattr(wl, "targets") else "dominant")
    bound = getattr(wl, "dom_bound", "hbm")
    if dom_ms <= 0:
        dom_ms = float("nan")                          # too few steps to reach the dominant kernel's turn
    if bound == "hbm":
        achieved, peak, unit = wl.dom_bytes / (dom_ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
    else:
        scale = 1e12 if wl.dom_unit == "TFLOP/s" else 1e9
        achieved, peak, unit = wl.dom_work / (dom_ms * 1e-3) / scale, wl.dom_peak, wl.dom_unit
    out = {
        "metric": "samples/sec for gather+sliced grad+reduce+SGD step; HBM GB/s and MFMA % of peak",
        "value": wl.units * steps / dt, "unit": wl.unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
        "warmup_steps_run": warmup + (0 if a.graph else warm_more), "repeats": repeats, "ms_per_step": dt / steps * 1e3,
        "ms_per_step_repeats": [t / steps * 1e3 for t in per_repeat], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.workload, "units_per_step": wl.units, "launch": "hip graph replay" if a.graph else "eager"},
        "roofline": {"bound": bound, "kernel": wl.dom_name, "achieved": achieved, "peak": peak,
                     "unit": unit, "frac": achieved / peak,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(a.config) if (a.rule == "momentum" and not a.collective and a.indexing == "list" and a.batch is None and not a.conv_shape and a.rows_per_worker is None) else None, "traffic_unit": "HBM bytes per launch",
                     "bytes_per_launch": wl.dom_bytes, "ms_per_launch": dom_ms,
                     "events_on_every_nth_step": timer.every, "launches_timed": timer.used},
    }
    if hasattr(wl, "mfmas_per_wave"):
        # the beside probe: a wavefront's MFMAs run one after the other, so the launch over their number is
        # the time per MFMA with the other instructions beside it
        out["roofline"]["ns_per_mfma_per_wavefront"] = dom_ms * 1e6 / wl.mfmas_per_wave
    if hasattr(wl, "kernel_report"):
        # every kernel of the step, timed on its own dispatches inside the timed region (one target a step,
        # rotating); the products against the matrix cores' peak for their input type, the streaming kernels
        # against HBM.  Targets of the task: >= 50 % of the bf16 peak for the gradient products, >= 70 % of HBM
        # for gather and reduce+update: `target_met` says whether this run reached them.
        ks = wl.kernel_report(timer)
        out["roofline"]["gemm"] = [dict(k, target_frac_mfma=0.5, target_met=k["frac_mfma"] >= 0.5)
                                   for k in ks if "flops" in k and k["kernel"] != "head"]
        out["roofline"]["kernels"] = [k for k in ks if "flops" not in k or k["kernel"] == "head"]
        step_bytes = sum(wl.kernel_work[k["kernel"]]["bytes"] for k in ks)
        gbs = step_bytes / (dt / steps) / 1e9
        out["roofline"]["step"] = {"bytes": step_bytes, "gbs": gbs, "frac_hbm": gbs / HBM_PEAK_GBS,
                                   "kernel_us_sum": sum(k["us"] for k in ks), "launches": len(ks)}
    if not a.no_cpu_baseline:
        from threadpoolctl import threadpool_limits
        v, sample = wl.cpu_baseline()
        cores = host_threads()
        with threadpool_limits(limits=1):
            v1, _ = wl.cpu_baseline()
        out["cpu_baseline"] = {"value": v, "unit": wl.unit, "cores": cores, "kind": "oracle",
                               "sample": sample, "value_1_thread": v1}
        out["context"] = "paper: 7.5x ResNet-50 speedup on 8x P100 (DGX-1) over 1 GPU; other hardware, not a target"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
