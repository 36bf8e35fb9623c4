"""Device-memory plumbing around the C ABI: allocate tensors and streams with PyTorch, lay the
seeded data out the way include/gacer.h specifies (channels-last activations, [cout][kh][kw][cin]
weights), fill the descriptor structs, and convert outputs back to logical NCHW.  No arithmetic
happens here; every operator runs inside libgacer.so.
"""
import ctypes as C

import numpy as np
import torch

from . import binding as B

_KIND = {"conv": B.GACER_CONV2D, "dwconv": B.GACER_DWCONV2D, "gemm": B.GACER_GEMM, "bgemm_qk": B.GACER_BGEMM_QK,
         "bgemm_pv": B.GACER_BGEMM_PV, "maxpool": B.GACER_MAXPOOL, "gavgpool": B.GACER_GAVGPOOL,
         "affine": B.GACER_AFFINE_ACT, "add": B.GACER_ADD, "layernorm": B.GACER_LAYERNORM,
         "softmax": B.GACER_SOFTMAX, "act": B.GACER_ACT, "scale": B.GACER_SCALE, "concat": B.GACER_CONCAT,
         "avgpool": B.GACER_AVGPOOL}
_ACT = {"none": B.GACER_ACT_NONE, "relu": B.GACER_ACT_RELU, "relu6": B.GACER_ACT_RELU6, "gelu": B.GACER_ACT_GELU,
        "hswish": B.GACER_ACT_HSWISH, "hsigmoid": B.GACER_ACT_HSIGMOID}
AXIS = {"none": B.GACER_AXIS_NONE, "batch": B.GACER_AXIS_BATCH, "cout": B.GACER_AXIS_COUT}
COUT_SPLITTABLE = ("conv", "dwconv", "gemm", "maxpool", "gavgpool", "affine", "scale", "concat", "avgpool")


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


class Session:
    """One gacer context with its tenants resident in HBM."""

    def __init__(self, tenants, data, device="cuda:0", shared_stream=False, place_streams=True):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: the library has no CPU fallback")
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.tenants = tenants
        self.ctx = C.c_void_p()
        B.check(self.ctx, B.gacer_create(C.byref(self.ctx)))
        self._keep = []
        self.streams = []
        self.sibling_streams = []
        place = place_streams and not shared_stream and len(tenants) > 1
        self.acts = []          # per tenant: list of device tensors (channels-last)
        descs = (B.gacer_tenant * len(tenants))()
        for ti, (t, (x, params)) in enumerate(zip(tenants, data)):
            tdt = torch.bfloat16 if t.dtype == "bf16" else torch.float32
            views = getattr(t, "views", {})
            acts = [None if i in views else torch.zeros((n, h, w, c), dtype=tdt, device=self.dev)
                    for i, (n, c, h, w) in enumerate(t.tensors)]
            for i, (base, off) in views.items():             # a channel window shares the wider tensor's storage
                acts[i] = acts[base][..., off:off + t.tensors[i][1]]
            acts[t.input].copy_(torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).to(tdt))
            self.acts.append(acts)
            tens = (B.gacer_tensor * len(acts))()
            for i, ((n, c, h, w), a) in enumerate(zip(t.tensors, acts)):
                base, off = views.get(i, (0, 0))
                tens[i] = B.gacer_tensor(n, c, h, w, a.data_ptr(), t.tensors[base][1] if i in views else 0, base, off)
            dev_params = {}

            def dparam(idx, kind=None, op=None):
                if idx < 0:
                    return None
                key = (idx, kind)
                if key not in dev_params:
                    a = params[idx]
                    if kind == "conv":
                        a = a.transpose(0, 2, 3, 1)                              # [O][I][kh][kw] -> [O][kh][kw][I]
                    elif kind == "dwconv":
                        a = a[:, 0].transpose(1, 2, 0)                           # [C][1][kh][kw] -> [kh][kw][C]
                    elif kind == "gemm_flat":
                        n, c, h, w = t.tensors[op.in0]
                        a = a.reshape(a.shape[0], c, h, w).transpose(0, 2, 3, 1)   # (c,h,w) -> (h,w,c) feature order
                    wdt = tdt if kind is not None else torch.float32
                    dev_params[key] = torch.from_numpy(np.ascontiguousarray(a)).to(wdt).to(self.dev).contiguous()
                return dev_params[key]

            ops = (B.gacer_op * len(t.ops))()
            for i, op in enumerate(t.ops):
                wkind = None
                if op.kind == "conv":
                    wkind = "conv"
                elif op.kind == "dwconv":
                    wkind = "dwconv"
                elif op.kind == "gemm":
                    n, c, h, w = t.tensors[op.in0]
                    wkind = "gemm_flat" if (op.cin != c and h * w > 1) else "gemm"
                alpha = op.eps if op.kind == "layernorm" else op.alpha
                ops[i] = B.gacer_op(_KIND[op.kind], op.in0, op.in1, op.res, op.out,
                                    _ptr(dparam(op.w, wkind, op)), _ptr(dparam(op.bias)), _ptr(dparam(op.scale)),
                                    _ptr(dparam(op.shift)), op.cin, op.cout, op.kh, op.kw, op.stride, op.pad,
                                    op.groups, _ACT[op.act], alpha)
            s = self.streams[0] if (shared_stream and self.streams) else torch.cuda.Stream(device=self.dev)
            self.streams.append(s)
            descs[ti] = B.gacer_tenant(len(t.ops), ops, len(acts), tens, t.input, t.output,
                                       B.GACER_BF16 if t.dtype == "bf16" else B.GACER_F32, t.batch,
                                       C.c_void_p(s.cuda_stream))
            self._keep += [tens, ops, dev_params]
        torch.cuda.synchronize(self.dev)
        if place:
            self._place_streams(descs, len(tenants))
        self._descs = descs
        B.check(self.ctx, B.gacer_load_tenants(self.ctx, descs, len(tenants)))

    # -- stream placement --------------------------------------------------------------------------
    def _place_streams(self, descs, n):
        """Hands 16 candidate streams to gacer_place_streams and gives every tenant the stream it chose (tenants spread
        over the device's hardware queues; see gacer_probe_stream_queues)."""
        cands = [torch.cuda.Stream(device=self.dev) for _ in range(16)]
        arr = (C.c_void_p * len(cands))(*[c.cuda_stream for c in cands])
        chosen, queue_of, nq, sib = (C.c_int * n)(), (C.c_int * n)(), C.c_int(), (C.c_int * n)()
        st = B.gacer_place_streams(descs, n, arr, len(cands), chosen, queue_of, C.byref(nq), sib)
        if st != B.GACER_OK:
            raise RuntimeError(f"gacer_place_streams failed with status {st}")
        self.queue_groups = nq.value
        self.tenant_queue = list(queue_of)
        self.streams = [cands[i] for i in chosen]
        self.sibling_streams = [cands[i] if i >= 0 else None for i in sib]
        for ti in range(n):
            descs[ti].stream = C.c_void_p(self.streams[ti].cuda_stream)
            if self.sibling_streams[ti] is not None:
                descs[ti].sibling_stream = C.c_void_p(self.sibling_streams[ti].cuda_stream)

    # -- plan ------------------------------------------------------------------------------------
    def set_plan(self, splits=(), syncs=()):
        """splits: iterable of (tenant, op, axis-name, factor) for even chunks, or (tenant, op, axis-name, [sizes...])
        for an explicit chunk list, each optionally followed by True to put the odd chunks on the tenant's sibling stream;
        syncs: (src_t, src_op, dst_t, dst_op[, when])."""
        rows, keep = [], []
        for row in splits:
            (t, o, a, f), sib = row[:4], (1 if len(row) > 4 and row[4] else 0)
            if isinstance(f, (list, tuple)):
                arr = (C.c_int * len(f))(*f)
                keep.append(arr)
                rows.append(B.gacer_split(t, o, AXIS[a], len(f), arr, sib))
            else:
                rows.append(B.gacer_split(t, o, AXIS[a], f, None, sib))
        sp = (B.gacer_split * max(1, len(rows)))(*rows)
        sy = (B.gacer_sync * max(1, len(syncs)))(*[B.gacer_sync(*e) for e in syncs])
        plan = B.gacer_plan(len(splits), sp, len(syncs), sy)
        B.check(self.ctx, B.gacer_set_plan(self.ctx, C.byref(plan)))

    def clear_plan(self):
        B.check(self.ctx, B.gacer_set_plan(self.ctx, None))

    def edges_from_pointers(self, matrix_P):
        n_ptr = len(matrix_P[0])
        flat = (C.c_int * max(1, len(matrix_P) * n_ptr))(*[p for P in matrix_P for p in P])
        out = C.POINTER(B.gacer_plan)()
        B.check(self.ctx, B.gacer_plan_from_pointers(self.ctx, flat, n_ptr, C.byref(out)))
        edges = [(out.contents.sync[i].src_tenant, out.contents.sync[i].src_op, out.contents.sync[i].dst_tenant,
                  out.contents.sync[i].dst_op, out.contents.sync[i].when) for i in range(out.contents.n_sync)]
        B.gacer_plan_free(out)
        return edges

    def uniform_splits(self, axis, factor, tenants=None):
        """Every operator that can be decomposed ``factor`` ways on ``axis`` (of the given tenants)."""
        out = []
        for ti, t in enumerate(self.tenants):
            if tenants is not None and ti not in tenants:
                continue
            for oi, op in enumerate(t.ops):
                if axis == "cout" and op.kind not in COUT_SPLITTABLE:
                    continue
                ext = t.batch if axis == "batch" else t.tensors[op.out][1]
                if factor <= ext:
                    out.append((ti, oi, axis, factor))
        return out

    # -- execution -------------------------------------------------------------------------------
    def run(self, mode=B.GACER_MODE_PLAN, rounds=1):
        ms = (C.c_float * rounds)()
        B.check(self.ctx, B.gacer_run(self.ctx, mode, rounds, ms))
        return list(ms)

    def run_static(self, mode=B.GACER_MODE_PLAN, rounds=1):
        """gacer_run_static: the same rounds with the split-K workspace inside the library (no allocation in the call)."""
        B.check(self.ctx, B.gacer_run_static(self.ctx, mode, rounds))

    def capture(self, mode=B.GACER_MODE_PLAN):
        """Capture one round of ``mode`` into a HIP graph; later run(mode) calls replay it."""
        B.check(self.ctx, B.gacer_capture(self.ctx, mode))

    def set_issue_threads(self, enable=True):
        """One host thread per tenant enqueues that tenant's stream (Section 2.1 deployment model)."""
        B.check(self.ctx, B.gacer_set_issue_threads(self.ctx, 1 if enable else 0))

    def set_fuse_affine(self, enable=True):
        """Affine + consuming 1x1 convolution as one launch where the plan allows (on by default)."""
        B.check(self.ctx, B.gacer_set_fuse_affine(self.ctx, 1 if enable else 0))

    def set_sync_every_launch(self, enable=True):
        """Checking mode: every kernel is waited for and checked before the next is issued."""
        B.check(self.ctx, B.gacer_set_sync_every_launch(self.ctx, 1 if enable else 0))

    def release_graphs(self):
        B.check(self.ctx, B.gacer_release_graphs(self.ctx))

    def issue_stats(self):
        """(host milliseconds spent enqueueing, operator launches enqueued) of the last run()."""
        ms, n = C.c_double(), C.c_int()
        B.check(self.ctx, B.gacer_issue_stats(self.ctx, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def launch_count(self, mode=B.GACER_MODE_PLAN):
        n = C.c_int()
        B.check(self.ctx, B.gacer_launch_count(self.ctx, mode, C.byref(n)))
        return n.value

    def trace(self, mode=B.GACER_MODE_PLAN, rounds=3):
        """Per-launch figures of one round (see gacer_trace_run)."""
        n = C.c_size_t()
        B.check(self.ctx, B.gacer_trace_run(self.ctx, mode, rounds, None, 0, C.byref(n)))
        rows = (B.gacer_launch_stat * n.value)()
        B.check(self.ctx, B.gacer_trace_run(self.ctx, mode, rounds, rows, n.value, C.byref(n)))
        return [dict(tenant=r.tenant, op=r.op, chunk=r.chunk, ms=r.ms, flops=r.flops, bytes=r.bytes,
                     workgroups=r.workgroups, kernel=r.kernel.decode(), start_ms=r.start_ms, end_ms=r.end_ms) for r in rows]

    def tensor(self, ti, idx):
        """Tensor ``idx`` of tenant ``ti`` as float32 numpy in logical NCHW order."""
        return self.acts[ti][idx].float().permute(0, 3, 1, 2).contiguous().cpu().numpy()

    def output(self, ti):
        return self.tensor(ti, self.tenants[ti].output)

    def output_bytes(self, ti):
        a = self.acts[ti][self.tenants[ti].output]
        return a.contiguous().view(torch.uint8).cpu().numpy().tobytes()

    def tensor_bytes(self, ti, idx):
        """Raw bytes of tensor ``idx`` of tenant ``ti`` as stored on the device."""
        return self.acts[ti][idx].contiguous().view(torch.uint8).cpu().numpy().tobytes()

    def poison_outputs(self):
        """Overwrite every non-input tensor with NaN so stale results cannot pass for fresh ones."""
        for t, acts in zip(self.tenants, self.acts):
            for i, a in enumerate(acts):
                if i != t.input:
                    a.fill_(float("nan"))
        torch.cuda.synchronize(self.dev)

    # -- lookup table and search -------------------------------------------------------------------
    def profile(self):
        n = C.c_size_t()
        B.check(self.ctx, B.gacer_profile(self.ctx, None, 0, C.byref(n)))
        rows = (B.gacer_prof * n.value)()
        B.check(self.ctx, B.gacer_profile(self.ctx, rows, n.value, C.byref(n)))
        return rows

    def search(self, rows, max_rounds=100):
        out = C.POINTER(B.gacer_plan)()
        ptrs = (C.c_int * (8 * len(self.tenants)))()
        n_ptr = C.c_int()
        R = C.c_double()
        B.check(self.ctx, B.gacer_search(self.ctx, rows, len(rows), max_rounds, C.byref(out), ptrs, C.byref(n_ptr), C.byref(R)))
        splits, syncs = self._plan_lists(out.contents)
        B.gacer_plan_free(out)
        P = [[ptrs[t * n_ptr.value + j] for j in range(n_ptr.value)] for t in range(len(self.tenants))]
        return splits, syncs, P, R.value

    def refine_plan(self, rows, rounds=12, min_gain=0.005):
        """gacer_refine on the installed plan; returns (splits, syncs, makespan_ms) of the refined, installed plan."""
        out = C.POINTER(B.gacer_plan)()
        ms = C.c_float()
        B.check(self.ctx, B.gacer_refine(self.ctx, rows, len(rows), rounds, min_gain, C.byref(out), C.byref(ms)))
        splits, syncs = self._plan_lists(out.contents)
        B.gacer_plan_free(out)
        return splits, syncs, ms.value

    @staticmethod
    def _plan_lists(pl):
        inv = {v: k for k, v in AXIS.items()}
        splits = []
        for i in range(pl.n_split):
            sp = pl.split[i]
            f = [sp.sizes[j] for j in range(sp.factor)] if sp.sizes else sp.factor
            splits.append((sp.tenant, sp.op, inv[sp.axis], f) + ((True,) if sp.sibling else ()))
        syncs = [(pl.sync[i].src_tenant, pl.sync[i].src_op, pl.sync[i].dst_tenant, pl.sync[i].dst_op, pl.sync[i].when)
                 for i in range(pl.n_sync)]
        return splits, syncs

    def close(self):
        if self.ctx:
            B.gacer_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
