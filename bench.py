#!/usr/bin/env python3
"""Benchmark of the sparse-graph-attention hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM: mask -> CSR (sga_build_mask, explicit workloads only) followed by
the fused attention forward (sga_attention_forward / sga_attention_forward_implicit).
The headline metric is attention edges per second (q.k pairs = H * NNZ per step).

Prints ONE JSON line.  `roofline` describes the attention forward (the dominant kernel), timed
live with events on the launch stream; `cpu_baseline` is the CPU oracle timed on a bounded
row sample of the same workload; `sweep` carries the other workloads (edges/s and ms/head
versus sequence length).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3    # dense fp32 MFMA
ALU_F32_PEAK_TFLOPS = 78.6      # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz (unpacked fp32 FMA)
kWarmSeconds = 0.05             # minimum untimed warm-up under load before the timed steps
FLOPS_PER_EDGE = 256            # 2d (q.k) + 2d (p*v accumulate), d = 64

# The largest single-GPU workload, and the one the >= 60 % HBM target is attached to.
DEFAULT_WORKLOAD = "cfg5_sliding_160m"

# HBM bytes per forward measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, written by
# `bench.py --traffic-summary` from the counter files of such runs (never edited by hand).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(name, prepared=False):
    """-> (bytes of the dominant kernel per launch, bytes of all kernels of one forward), or
    (None, None) where no counter run is on file."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(name + ("/prepared" if prepared else ""))
    except (OSError, ValueError):
        rec = None
    if not rec:
        return None, None
    return rec.get("dominant_kernel_bytes"), rec.get("forward_bytes")


def tensor_bytes(wl):
    """Q, K, V read once and O written once: 4*d*sizeof per row and head."""
    return 4 * wl.d * (4 if wl.dtype == "f32" else 2) * wl.L * wl.H


def algorithmic_bytes(wl, nnz):
    """Compulsory HBM bytes of one forward: Q, K, V read once and O written once
    (4*d*sizeof per row and head) plus, for explicit masks, col_idx (4 B/edge) and
    row_ptr (8 B/row) read once for all heads."""
    b = tensor_bytes(wl)
    if wl.explicit:
        b += 4 * nnz + 8 * (wl.L + 1)
    return b


class Runner:
    """Holds device buffers of one workload and runs steps."""

    def __init__(self, wl, path):
        import torch
        import paper_2502_01659_amd as sga
        from sga_inputs import torch_qkv
        self.torch, self.sga, self.wl, self.path = torch, sga, wl, path
        dev = "cuda:0"
        self.random = wl.mask.name == "random"      # CSR drawn once; no builder call per step
        if self.random:
            from sga_inputs import torch_random_csr
            self.row_ptr, self.col_idx = torch_random_csr(wl.mask, dev)
            self.nnz = int(self.row_ptr[-1])
        else:
            self.nnz = sga.mask_nnz(wl.mask)
        self.Q, self.K, self.V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, dev)
        self.O = torch.empty_like(self.Q)
        if wl.explicit and not self.random:
            self.row_ptr = torch.empty(wl.L + 1, dtype=torch.int64, device=dev)
            self.col_idx = torch.empty(self.nnz, dtype=torch.int32, device=dev)
        self.ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, self.nnz if wl.explicit else -1,
                                      device=dev)
        self.stream = torch.cuda.current_stream().cuda_stream
        self.dt = 0 if wl.dtype == "f32" else 1
        self.plan = None            # prepared graph (explicit workloads, see prepare())
        self.prepared = False       # steps run the prepared forward only

    def prepare(self):
        """Mask -> CSR -> tile graph once; later steps reuse it (sga_attention_forward_prepared)."""
        self.build()
        st, self.plan = self.sga.sga_graph_prepare(self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                                                   self.wl.L, self.wl.H, self.wl.d, self.dt,
                                                   self.ws.data_ptr(), self.ws.numel(), self.stream)
        if st != 0:
            raise self.sga.SgaError(st, "sga_graph_prepare")
        self.prepared = True

    def build(self):
        if self.random:
            return
        st = self.sga.sga_build_mask(self.wl.mask, self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                                     self.col_idx.numel(), self.stream)
        if st != 0:
            raise self.sga.SgaError(st, "sga_build_mask")

    def forward(self):
        wl, sga = self.wl, self.sga
        if self.prepared:
            st = sga.sga_attention_forward_prepared(self.Q.data_ptr(), self.K.data_ptr(), self.V.data_ptr(),
                                                    self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                                                    self.O.data_ptr(), wl.L, wl.H, wl.d, wl.scale,
                                                    self.stream, self.dt, None, self.ws.data_ptr(),
                                                    self.ws.numel(), self.path, self.plan)
        elif wl.explicit:
            st = sga.sga_attention_forward(self.Q.data_ptr(), self.K.data_ptr(), self.V.data_ptr(),
                                           self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                                           self.O.data_ptr(), wl.L, wl.H, wl.d, wl.scale, self.stream,
                                           self.dt, None, self.ws.data_ptr(), self.ws.numel(), self.path)
        else:
            st = sga.sga_attention_forward_implicit(self.Q.data_ptr(), self.K.data_ptr(),
                                                    self.V.data_ptr(), wl.mask, self.O.data_ptr(),
                                                    wl.L, wl.H, wl.d, wl.scale, self.stream, self.dt,
                                                    None, self.ws.data_ptr(), self.ws.numel(), self.path)
        if st != 0:
            raise sga.SgaError(st, "sga_attention_forward")

    def step(self):
        if self.wl.explicit and not self.prepared:
            self.build()
        self.forward()

    def timed(self, steps, warmup):
        """-> (wall ms per step, mean forward ms, mean build ms, mean dominant-kernel ms).

        The step time is the wall clock over exactly `steps` steps between two device
        synchronisations; the only instrumentation inside that region is the library's own event
        pair around the fused attention kernel of each forward (sga_profile_*, on the launch
        stream), which gives the dominant-kernel time.  The split into mask build and forward
        comes from a second pass of the same steps with events around the two C-ABI calls (each
        event record costs about 5 us on the stream, so it is kept out of the timed region)."""
        torch = self.torch
        # Untimed warm-up: at least `warmup` steps, and at least kWarmSeconds of device time.  The
        # device reaches its sustained clock only after some tens of milliseconds under load: the
        # paper's 10 warm-up launches are 6 ms of workload 2 and end while it is still ramping up
        # (the kernel then reads 0.52 ms instead of 0.48 ms).
        done = 0
        t_warm = time.perf_counter()
        while done < warmup or time.perf_counter() - t_warm < kWarmSeconds:
            self.step()
            done += 1
            if done % 8 == 0 or done >= warmup:
                torch.cuda.synchronize()
        self.warmup_steps_run = done
        torch.cuda.synchronize()
        self.sga.sga_profile_enable(1)
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st, kern = self.sga.sga_profile_collect(steps)
        kernel_name_ = self.sga.sga_profile_last_kernel()
        self.sga.sga_profile_enable(0)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for k in range(steps):
            ev[k][0].record()
            if self.wl.explicit and not self.prepared:
                self.build()
            ev[k][1].record()
            self.forward()
            ev[k][2].record()
        torch.cuda.synchronize()
        fwds = [e[1].elapsed_time(e[2]) for e in ev]
        fwd = sum(fwds) / steps
        bld = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
        kern_ms = sum(kern) / len(kern) if st == 0 and kern else fwd
        self.kernel = kernel_name_ if st == 0 and kern else "forward (no event pair)"
        # fastest single launch (the paper's protocol reports mean and min)
        self.min_forward_ms = min(fwds)
        self.min_kernel_ms = min(kern) if st == 0 and kern else min(fwds)
        return (t1 - t0) * 1e3 / steps, fwd, bld, kern_ms

    def cold(self, launches=5):
        """Forward with the caches emptied first: a 1 GiB buffer (four times the 256 MB
        last-level cache) is overwritten before every launch.  -> (mean forward ms, mean
        dominant-kernel ms).  Meaningful for the workloads whose tensors fit that cache."""
        torch = self.torch
        scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        if self.wl.explicit and not self.prepared:
            self.build()
        self.sga.sga_profile_enable(1)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(launches)]
        for k in range(launches):
            scratch.fill_(k)
            ev[k][0].record()
            self.forward()
            ev[k][1].record()
        torch.cuda.synchronize()
        st, kern = self.sga.sga_profile_collect(launches)
        self.sga.sga_profile_enable(0)
        del scratch
        fwd = sum(e[0].elapsed_time(e[1]) for e in ev) / launches
        return fwd, (sum(kern) / len(kern) if st == 0 and kern else fwd)


def gather_aware_bytes(wl, nnz, prepared=False):
    """Algorithmic bytes plus the K/V rows that no reuse can save: in the BigBird-style mask every
    non-global query block row fetches its random key blocks (K and V) for itself, and the global
    query rows pass over all of K and V once more per head.  Equal to the algorithmic bytes for
    the other masks."""
    b = tensor_bytes(wl) if prepared else algorithmic_bytes(wl, nnz)
    m = wl.mask
    if m.name == "bigbird":
        size = 4 if wl.dtype == "f32" else 2
        nb = wl.L // m.block
        per_head = (nb - m.n_global_blocks) * m.n_random_blocks * m.block * wl.d * size * 2
        if m.n_global_blocks > 0:
            per_head += 2 * wl.L * wl.d * size
        b += wl.H * per_head
    return b


def roofline_of(wl, nnz, kern_ms, fwd_ms, path_used, kernel, prepared=False):
    """Roofline of the dominant kernel (the fused attention kernel) from its own duration, and
    the same at the level of the whole forward call.

    Dominant kernel: `achieved` counts only what that kernel touches -- for fp16 storage the
    tensor bytes (Q, K, V read once, O written once; the tile kernel of an explicit mask reads
    the tile graph, not col_idx, so no index bytes are counted for it), for fp32 storage the
    256 flops per edge.  Forward level (`forward`): the algorithmic bytes of the call (tensor
    bytes plus, for an unprepared explicit call, 4 B per edge of col_idx and 8 B per row of
    row_ptr) and the same flops, over the duration of the whole call."""
    edges = nnz * wl.H
    t, tf = kern_ms * 1e-3, fwd_ms * 1e-3
    split = path_used == "tile_split"
    # (the per-row kernels do their products on the vector unit, whichever path was asked for)
    path_used = "gather" if path_used == "gather" or str(kernel).startswith("gather") else "tile"
    flops = FLOPS_PER_EDGE * edges
    kbytes = tensor_bytes(wl)
    fbytes = kbytes if prepared else algorithmic_bytes(wl, nnz)
    if wl.dtype == "f32" and not split:
        bound, peak = ("alu", ALU_F32_PEAK_TFLOPS) if path_used == "gather" else ("mfma", MFMA_F32_PEAK_TFLOPS)
        ach, ach_f, unit = flops / t / 1e12, flops / tf / 1e12, "TFLOP/s"
    else:
        # fp16 storage, and fp32 storage on the split-precision path (three fp16 matrix-core
        # products per product: 0.12 PFLOP at workload 2, 46 us at the fp16 peak, below the
        # 77 us the compulsory bytes take): bound by HBM
        bound, peak, unit = "hbm", HBM_PEAK_GBPS, "GB/s"
        ach, ach_f = kbytes / t / 1e9, fbytes / tf / 1e9
    traffic_kernel, traffic_forward = measured_traffic(wl.name, prepared)
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
            "traffic": traffic_kernel,
            "kernel": kernel, "kernel_ms": kern_ms,
            "kernel_bytes": kbytes, "kernel_hbm_GBps": kbytes / t / 1e9,
            "algorithmic_flops": flops,
            "forward": {"ms": fwd_ms, "achieved": ach_f, "unit": unit, "frac": ach_f / peak,
                        "algorithmic_bytes": fbytes, "hbm_GBps": fbytes / tf / 1e9,
                        "hbm_frac": fbytes / tf / 1e9 / HBM_PEAK_GBPS, "traffic": traffic_forward},
            "gather_aware_bytes": gather_aware_bytes(wl, nnz, prepared),
            "hbm_gather_aware_GBps": gather_aware_bytes(wl, nnz, prepared) / t / 1e9}


def cpu_baseline(wl, runner, budget_s=12.0, target_s=1.5):
    """The oracle (row scan over all keys, two-pass softmax, float64) on a bounded row sample
    of the same workload, on the host cores of this machine: seeded random rows of head 0 and, if
    the whole head takes less than target_s, of the following heads (about 20 core-seconds)."""
    import numpy as np
    from oracle import rowscan
    torch = runner.torch
    threads = rowscan.num_threads()
    rng = np.random.default_rng(wl.seed + 4)
    spec = wl.mask
    if wl.L <= (1 << 21):
        def run(head, rows):
            Qh = runner.Q[head].float().cpu().numpy()
            Kh = runner.K[head].float().cpu().numpy()
            Vh = runner.V[head].float().cpu().numpy()
            t0 = time.perf_counter()
            _, _, edges = rowscan.attend_rows(spec, Qh, Kh, Vh, wl.scale, rows)
            return time.perf_counter() - t0, edges
    else:
        def run(head, rows):
            # K/V stay on the device; only the neighbours' rows are fetched.  The predicate scans
            # (one per row, all L keys each) are spread over the host cores, one row per thread.
            from concurrent.futures import ThreadPoolExecutor
            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=threads) as pool:
                lists = list(pool.map(lambda i: rowscan.row_neighbors(spec, int(i)), rows))
            edges = 0
            q = runner.Q[head][torch.from_numpy(rows).cuda()].float().cpu().numpy()
            for r, nb in enumerate(lists):
                idx = torch.from_numpy(nb).cuda()
                Kg = runner.K[head][idx].float().cpu().numpy()
                Vg = runner.V[head][idx].float().cpu().numpy()
                rowscan.attend_gathered(q[r], Kg, Vg, wl.scale)
                edges += len(nb)
            return time.perf_counter() - t0, edges
    probe = np.sort(rng.choice(wl.L, size=min(wl.L, (8 if wl.L <= (1 << 21) else 1) * threads),
                               replace=False)).astype(np.int64)
    t_probe, _ = run(0, probe)
    per_row = max(t_probe / len(probe), 1e-7)
    n = int(min(wl.L, max(len(probe), budget_s / per_row)))
    rows = np.sort(rng.choice(wl.L, size=n, replace=False)).astype(np.int64)
    t, edges = run(0, rows)
    for _ in range(2):          # the probe rows pay for the first touches: top the sample up to the budget
        if n == wl.L or t >= 0.8 * budget_s:
            break
        more = np.setdiff1d(rng.choice(wl.L, size=min(wl.L, int(n * (budget_s - t) / t) + 1), replace=False), rows)
        if len(more) == 0:
            break
        dt, de = run(0, more.astype(np.int64))
        rows = np.union1d(rows, more).astype(np.int64)
        t, edges, n = t + dt, edges + de, len(rows)
    heads, n_rows = 1, n
    while n == wl.L and t < target_s and heads < wl.H:      # whole heads were cheap: take more
        dt, de = run(heads, rows)
        t, edges, heads, n_rows = t + dt, edges + de, heads + 1, n_rows + n
    return {"value": edges / t, "unit": "edges/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} seeded random query rows of each of the first {heads} head(s) of {wl.name} "
                      f"(each row scans all {wl.L} keys through the mask predicate), {edges} edges in "
                      f"{t:.2f} s of oracle time",
            "seconds": t, "us_per_row": t / n_rows * 1e6,
            "extrapolated_full_workload_s": t / n_rows * wl.L * wl.H}


def composition_times(wl, path, steps=5, warmup=2):
    """Section V-F's comparison on the headline mask: one CSR call on the global+local mask
    against a local call followed by a global (non-local) call on the same (O, lse) state."""
    import torch
    import paper_2502_01659_amd as sga
    from sga_inputs import MaskSpec, KIND_SLIDING, KIND_NONLOCAL, torch_qkv
    m = wl.mask
    loc = MaskSpec(KIND_SLIDING, wl.L, window=m.window)
    nl = MaskSpec(KIND_NONLOCAL, wl.L, window=m.window, n_global=m.n_global)
    Q, K, V = torch_qkv(wl.H, wl.L, wl.d, wl.dtype, wl.sigma, wl.seed, "cuda:0")
    O = torch.empty_like(Q)
    lse = torch.empty((wl.H, wl.L), dtype=torch.float32, device="cuda:0")
    rp, ci = sga.build_mask(m)
    rp1, ci1 = sga.build_mask(loc)
    rp2, ci2 = sga.build_mask(nl)
    ws = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp[-1]))
    ws1 = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp1[-1]))
    ws2 = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, int(rp2[-1]))
    wsi = sga.alloc_workspace(wl.L, wl.H, wl.d, wl.dtype, -1)

    def single():
        sga.attention_forward(Q, K, V, rp, ci, wl.scale, O=O, lse=lse, workspace=ws, path=path)

    def implicit_pair():
        sga.attention_forward_implicit(Q, K, V, loc, wl.scale, O=O, lse=lse, workspace=wsi, path=path)
        sga.attention_accumulate_implicit(Q, K, V, nl, wl.scale, O, lse, workspace=wsi, path=path)

    def csr_pair():
        sga.attention_forward(Q, K, V, rp1, ci1, wl.scale, O=O, lse=lse, workspace=ws1, path=path)
        sga.attention_accumulate(Q, K, V, rp2, ci2, wl.scale, O, lse, workspace=ws2, path=path)

    out = {}
    for name, fn in (("single_csr_ms", single), ("local_then_nonlocal_implicit_ms", implicit_pair),
                     ("local_then_nonlocal_csr_ms", csr_pair)):
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / steps
    out["mask"] = f"window {m.window} + {m.n_global} global tokens, L={wl.L}, H={wl.H}, {wl.dtype}"
    return out


def _time_calls(fn, steps, warmup):
    import torch
    done, t_warm = 0, time.perf_counter()
    while done < warmup or time.perf_counter() - t_warm < kWarmSeconds / 2:   # (see Runner.timed)
        fn()
        done += 1
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def suite_table3(path):
    """The long-context shapes of the paper's Table III (Section V-E): local attention, fp16,
    one head, window sized to S_f = 2730/L (S_f = 1e-5 at 160M tokens).  The paper's A100
    seconds are quoted beside ours as context (another machine, another implementation)."""
    import torch
    import paper_2502_01659_amd as sga
    from sga_inputs import MaskSpec, KIND_SLIDING, torch_qkv, BASE_SEED
    shapes = [(1_600_000, 0.0017, 12.46), (8_000_000, 0.00034, 62.32), (16_000_000, 0.00017, 124.67),
              (160_000_000, 0.00001, 733.93)]
    rows = []
    for L, sf, paper_s in shapes:
        w = max(0, (int(round(sf * L)) - 1) // 2)
        spec = MaskSpec(KIND_SLIDING, L, window=w)
        Q, K, V = torch_qkv(1, L, 64, "f16", 0.5, BASE_SEED, "cuda:0")
        O = torch.empty_like(Q)
        ms = _time_calls(lambda: sga.attention_forward_implicit(Q, K, V, spec, 0.125, O=O, path=path),
                         steps=3, warmup=1)
        edges = sga.mask_nnz(spec)
        rows.append({"L": L, "window": w, "S_f": edges / (L * L), "edges": edges, "dtype": "f16", "d": 64,
                     "ms": ms, "edges_per_s": edges / (ms * 1e-3),
                     "hbm_algorithmic_GBps": 4 * L * 64 * 2 / (ms * 1e-3) / 1e9,
                     "mfma_f16_TFLOPs": FLOPS_PER_EDGE * edges / (ms * 1e-3) / 1e12,
                     "paper_a100_seconds": paper_s, "paper_over_ours": paper_s * 1e3 / ms})
        del Q, K, V, O
        torch.cuda.empty_cache()
    return {"suite": "table3", "unit": "ms per forward (sga_attention_forward_implicit)", "rows": rows}


def suite_d128(path, n_shapes=5):
    """Sliding windows at d = 128, fp16, the head size of the models in the paper's table of
    context limits (Section V-D) and of most current ones: wide bands (matrix-core regime) and
    narrow windows (HBM regime), implicit neighbours."""
    import torch
    import paper_2502_01659_amd as sga
    from sga_inputs import MaskSpec, KIND_SLIDING, KIND_DILATED, torch_qkv, BASE_SEED
    rows = []
    for L, H, w, s in ((32768, 32, 2048, 1), (131072, 8, 1024, 1), (32768, 32, 256, 1),
                       (1 << 20, 4, 64, 2), (1 << 20, 4, 16, 1))[:n_shapes]:
        spec = MaskSpec(KIND_DILATED if s > 1 else KIND_SLIDING, L, window=w, stride=s)
        Q, K, V = torch_qkv(H, L, 128, "f16", 0.5, BASE_SEED, "cuda:0")
        O = torch.empty_like(Q)
        ws = sga.alloc_workspace(L, H, 128, "f16", -1)
        ms = _time_calls(lambda: sga.attention_forward_implicit(Q, K, V, spec, 128 ** -0.5, O=O, workspace=ws,
                                                                path=path), steps=10, warmup=3)
        edges = sga.mask_nnz(spec) * H
        rows.append({"L": L, "H": H, "d": 128, "window": w, "stride": s, "dtype": "f16", "edges": edges, "ms": ms,
                     "edges_per_s": edges / (ms * 1e-3),
                     "hbm_algorithmic_GBps": 4 * L * H * 128 * 2 / (ms * 1e-3) / 1e9,
                     "mfma_f16_TFLOPs": 4.0 * 128 * edges / (ms * 1e-3) / 1e12})
        del Q, K, V, O, ws
        torch.cuda.empty_cache()
    # explicit masks at the same head size, on a prepared graph: workload 4's and workload 2's masks
    # and a +-512 window handed over as CSR
    if n_shapes >= 5:
        from sga_inputs import WORKLOADS
        for name, spec, H in (("cfg4 mask", WORKLOADS["cfg4_bigbird_1m"].mask, 4),
                              ("cfg2 mask", WORKLOADS["cfg2_longformer_64k"].mask, 8),
                              ("sliding +-512 as CSR", MaskSpec(KIND_SLIDING, 1 << 18, window=512), 4)):
            rp, ci = sga.build_mask(spec)
            nnz = int(rp[-1])
            Q, K, V = torch_qkv(H, spec.L, 128, "f16", 0.5, BASE_SEED, "cuda:0")
            O = torch.empty_like(Q)
            ws = sga.alloc_workspace(spec.L, H, 128, "f16", nnz)
            plan = sga.graph_prepare(rp, ci, H, 128, "f16", ws)
            ms = _time_calls(lambda: sga.attention_forward_prepared(Q, K, V, rp, ci, 128 ** -0.5, plan, ws, O=O),
                             steps=10, warmup=3)
            rows.append({"mask": name, "entry": "csr, prepared graph", "L": spec.L, "H": H, "d": 128, "dtype": "f16",
                         "edges": nnz * H, "ms": ms, "edges_per_s": nnz * H / (ms * 1e-3),
                         "hbm_algorithmic_GBps": 4 * spec.L * H * 128 * 2 / (ms * 1e-3) / 1e9,
                         "mfma_f16_TFLOPs": 4.0 * 128 * nnz * H / (ms * 1e-3) / 1e12})
            del Q, K, V, O, ws, rp, ci
            torch.cuda.empty_cache()
    return {"suite": "d128", "unit": "ms per forward (implicit windows, then explicit masks on prepared graphs)",
            "rows": rows}


def suite_e2(path, dims=(64, 128, 256)):
    """The shapes of the paper's microbenchmark (Section V-C): L in {8192, 16384, 24576}, one
    head, fp32, sparsity factors across (0, 1], masks sized to the sparsity factor: local,
    1-D dilated (r = 1), 2-D dilated (r = 1), global with the smallest local window, and a
    uniformly random CSR mask."""
    import torch
    import paper_2502_01659_amd as sga
    from sga_inputs import (MaskSpec, KIND_SLIDING, KIND_DILATED, KIND_DILATED_2D, KIND_GLOBAL_LOCAL,
                            torch_qkv, BASE_SEED)
    rows = []
    for d in dims:
        for L in (8192, 16384, 24576):
            Q, K, V = torch_qkv(1, L, d, "f32", 1.0, BASE_SEED, "cuda:0")
            O = torch.empty_like(Q)
            for sf in (0.001, 0.01, 0.1, 0.5, 1.0):
                span = max(1, int(round(sf * L)))
                specs = {
                    "local": MaskSpec(KIND_SLIDING, L, window=(span - 1) // 2),
                    "dilated_1d": MaskSpec(KIND_DILATED, L, window=(span - 1) // 2, stride=2),
                    "dilated_2d": MaskSpec(KIND_DILATED_2D, L, block=min(L, max(2, 4 * span)), stride=2),
                    "global": MaskSpec(KIND_GLOBAL_LOCAL, L, window=0, n_global=min(L, max(1, span // 2))),
                }
                for name, spec in specs.items():
                    implicit = name != "global"
                    if implicit:
                        wsi = sga.alloc_workspace(L, 1, d, "f32", -1)
                        fn = lambda: sga.attention_forward_implicit(Q, K, V, spec, d ** -0.5, O=O,
                                                                    workspace=wsi, path=path)
                        edges = sga.mask_nnz(spec)
                    else:
                        rp, ci = sga.build_mask(spec)
                        edges = int(rp[-1])
                        ws = sga.alloc_workspace(L, 1, d, "f32", edges)
                        fn = lambda: sga.attention_forward(Q, K, V, rp, ci, d ** -0.5, O=O, workspace=ws,
                                                           path=path)
                    ms = _time_calls(fn, steps=5, warmup=2)
                    rows.append({"mask": name, "entry": "implicit" if implicit else "csr", "L": L, "d": d,
                                 "S_f_target": sf, "S_f": edges / (L * L), "edges": edges, "ms": ms,
                                 "edges_per_s": edges / (ms * 1e-3)})
                # uniformly random explicit mask
                g = torch.Generator(device="cuda:0")
                g.manual_seed(BASE_SEED + 7)
                dense = torch.rand((L, L), generator=g, device="cuda:0") < sf
                rp = torch.zeros(L + 1, dtype=torch.int64, device="cuda:0")
                rp[1:] = dense.sum(dim=1).cumsum(0)
                ci = dense.nonzero()[:, 1].to(torch.int32).contiguous()
                del dense
                edges = int(rp[-1])
                ws = sga.alloc_workspace(L, 1, d, "f32", edges)
                ms = _time_calls(lambda: sga.attention_forward(Q, K, V, rp, ci, d ** -0.5, O=O,
                                                               workspace=ws, path=path), steps=5, warmup=2)
                rows.append({"mask": "random_csr", "entry": "csr", "L": L, "d": d, "S_f_target": sf,
                             "S_f": edges / (L * L), "edges": edges, "ms": ms,
                             "edges_per_s": edges / (ms * 1e-3)})
                del rp, ci, ws
                torch.cuda.empty_cache()
            del Q, K, V, O
    return {"suite": "e2", "unit": "ms per forward, one head, fp32", "rows": rows}


def suite_vf(path, dtype="f32"):
    """The masks of the paper's model comparison (Section V-F): local attention of 50 tokens each
    way with three global tokens (Longformer), the same with a dilated window (every second
    token, 100 each way), and local + global + uniformly random attention at S_f = 0.001
    (BigBird), one head, d = 64, four context lengths.  Each mask runs as one CSR call (first
    call and prepared graph); the first and the third also as the paper's sequence of calls on
    one (O, lse) state: implicit local, implicit global (non-local), and for the third a CSR call
    on the random edges that the first two do not cover.  The two forms are compared (largest
    difference of O) as the paper does."""
    import torch
    import paper_2502_01659_amd as sga
    from sga_inputs import MaskSpec, KIND_SLIDING, KIND_NONLOCAL, KIND_GLOBAL_LOCAL, torch_qkv, BASE_SEED
    w, g, d, sf = 50, 3, 64, 0.001
    scale = d ** -0.5
    rows = []

    def csr_of(dense):
        rp = torch.zeros(dense.shape[0] + 1, dtype=torch.int64, device="cuda:0")
        rp[1:] = dense.sum(dim=1).cumsum(0)
        # (row blocks: one nonzero() over more than 2^31 entries is beyond the library routine)
        cols = [dense[r0:r0 + 4096].nonzero()[:, 1].to(torch.int32) for r0 in range(0, dense.shape[0], 4096)]
        return rp, torch.cat(cols).contiguous()

    for L in (10_000, 20_000, 35_000, 50_000):
        Q, K, V = torch_qkv(1, L, d, dtype, 1.0 if dtype == "f32" else 0.5, BASE_SEED, "cuda:0")
        loc = MaskSpec(KIND_SLIDING, L, window=w)
        nl = MaskSpec(KIND_NONLOCAL, L, window=w, n_global=g)
        i = torch.arange(L, device="cuda:0")[:, None]
        j = torch.arange(L, device="cuda:0")[None, :]
        glob = (i < g) | (j < g)
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(BASE_SEED + 11)
        rand = torch.rand((L, L), generator=gen, device="cuda:0") < sf
        longformer = ((i - j).abs() <= w) | glob
        masks = {
            "longformer": (longformer, (loc, nl, None)),
            "longformer_dilated": ((((i - j).abs() <= 2 * w) & ((i - j) % 2 == 0)) | glob, None),
            "bigbird": (longformer | rand, (loc, nl, rand & ~longformer)),
        }
        del glob
        wsi = sga.alloc_workspace(L, 1, d, dtype, -1)
        for name, (dense, parts) in masks.items():
            rp, ci = csr_of(dense)
            del dense
            edges = int(rp[-1])
            ws = sga.alloc_workspace(L, 1, d, dtype, edges)
            O1 = torch.empty_like(Q)
            ms_csr = _time_calls(lambda: sga.attention_forward(Q, K, V, rp, ci, scale, O=O1, workspace=ws, path=path),
                                 steps=15, warmup=10)
            plan = sga.graph_prepare(rp, ci, 1, d, dtype, ws)
            ms_prep = _time_calls(lambda: sga.attention_forward_prepared(Q, K, V, rp, ci, scale, plan, ws, O=O1),
                                  steps=15, warmup=10)
            row = {"mask": name, "L": L, "d": d, "dtype": dtype, "edges": edges, "S_f": edges / (L * L),
                   "csr_ms": ms_csr, "csr_prepared_ms": ms_prep, "edges_per_s": edges / (ms_prep * 1e-3)}
            if parts is not None:
                p_loc, p_nl, extra = parts
                O2 = torch.empty_like(Q)
                lse = torch.empty((1, L), dtype=torch.float32, device="cuda:0")
                if extra is not None:
                    rp3, ci3 = csr_of(extra)
                    ws3 = sga.alloc_workspace(L, 1, d, dtype, int(rp3[-1]))

                def sequence():
                    sga.attention_forward_implicit(Q, K, V, p_loc, scale, O=O2, lse=lse, workspace=wsi, path=path)
                    sga.attention_accumulate_implicit(Q, K, V, p_nl, scale, O2, lse, workspace=wsi, path=path)
                    if extra is not None:
                        sga.attention_accumulate(Q, K, V, rp3, ci3, scale, O2, lse, workspace=ws3, path=path)
                row["sequence_ms"] = _time_calls(sequence, steps=15, warmup=10)
                row["sequence_calls"] = 2 if extra is None else 3
                torch.cuda.synchronize()
                row["max_abs_difference"] = (O1.float() - O2.float()).abs().max().item()
            rows.append(row)
            del rp, ci, ws
            torch.cuda.empty_cache()
        del masks, rand, longformer, Q, K, V
        torch.cuda.empty_cache()
    return {"suite": "vf", "unit": "ms per forward, one head, d = 64, " + dtype, "rows": rows}


def fits_cache(wl):
    """One head's Q, K, V, O fit the 256 MB last-level cache."""
    return 4 * wl.d * (4 if wl.dtype == "f32" else 2) * wl.L <= (256 << 20)


def steady_state(run, steps, warmup, path_name):
    """Explicit workloads with the mask fixed across steps (the masks of Section II-C are static
    patterns): CSR built and tile graph prepared once, then sga_attention_forward_prepared per
    step.  -> forward and kernel times and the roofline figures of that forward."""
    run.prepare()
    ms, f, _, km = run.timed(steps, warmup)
    wl = run.wl
    p = run.plan
    return {"step": "sga_attention_forward_prepared (sga_build_mask + sga_graph_prepare once, untimed)",
            "ms_per_step": ms, "forward_ms": f, "forward_ms_min": run.min_forward_ms, "kernel_ms": km,
            "forward_edges_per_s": run.nnz * wl.H / (f * 1e-3),
            "plan": {"tiles_left": p.tiles_left, "multi_tiles": p.multi_tiles, "tile_parts": p.tile_parts,
                     "long_rows": p.long_rows, "flags": p.flags},
            "roofline": roofline_of(wl, run.nnz, km, f, path_name, run.kernel, prepared=True)}


def _kernel_label(name):
    """Short label of a kernel in a rocprofv3 csv: sga kernels by name and storage type, the copy
    kernel of --calibrate-copy as 'copy', others None."""
    import re
    m = re.search(r"sga::\(anonymous namespace\)::(\w+)", name) or re.search(r"sga::(\w+)", name)
    if m:
        kind = "<half>" if "__half" in name else "<float>" if "<float" in name else ""
        return m.group(1) + kind
    if "copyBuffer" in name or "direct_copy" in name:     # the runtime's device-to-device copy kernel
        return "copy"
    return None


def _counter_per_kernel(csv_path):
    """-> {label: (dispatches, summed counter value in KiB)} of one rocprofv3 --pmc csv."""
    import csv
    out = {}
    with open(csv_path, newline="") as f:
        for row in csv.DictReader(f):
            lab = _kernel_label(row["Kernel_Name"])
            if lab is None:
                continue
            n, v = out.get(lab, (0, 0.0))
            out[lab] = (n + 1, v + float(row["Counter_Value"]))
    return out


def traffic_summary(dir_, workload, prepared):
    """Per-kernel HBM bytes of one forward from four rocprofv3 --pmc runs under `dir_`:
    fetch_<tag>/, write_<tag>/ (bench.py --workload ... on FETCH_SIZE, then WRITE_SIZE) and
    fetch_copy/, write_copy/ (bench.py --calibrate-copy: a plain 1 GiB device copy), each holding
    one *_counter_collection.csv.  The copy fixes the scale of either counter (bytes per KiB
    read).  Prints a table, and records the totals under profiles/hbm_traffic.json."""
    import glob
    tag = workload + ("_prepared" if prepared else "")

    def load(sub):
        files = glob.glob(os.path.join(dir_, sub, "**", "*counter_collection.csv"), recursive=True)
        if len(files) != 1:
            raise SystemExit(f"expected one counter csv under {dir_}/{sub}, found {len(files)}")
        return _counter_per_kernel(files[0])

    cal = {}
    for which in ("fetch", "write"):
        n, kib = load(f"{which}_copy")["copy"]
        cal[which] = (1 << 30) / (kib / n * 1024.0)      # bytes moved per byte the counter shows
    fetch, write = load(f"fetch_{tag}"), load(f"write_{tag}")
    attend = [k for k in fetch if k.startswith(("tile_attend", "tile_window", "gather_csr", "gather_window"))]
    dominant = max(attend, key=lambda k: fetch[k][1] + write.get(k, (0, 0))[1])
    steps = fetch[dominant][0]
    rows, total = [], 0.0
    for k in sorted(fetch, key=lambda k: -(fetch[k][1] + write.get(k, (0, 0))[1])):
        if k == "copy" or k == "build_mask_kernel":
            continue
        rd = fetch[k][1] * 1024.0 * cal["fetch"] / steps
        wr = write.get(k, (0, 0.0))[1] * 1024.0 * cal["write"] / steps
        rows.append((k, fetch[k][0] / steps, rd, wr))
        total += rd + wr
    dom = next(r for r in rows if r[0] == dominant)
    print(f"HBM traffic per forward of {tag} (FETCH_SIZE x {cal['fetch']:.3f}, WRITE_SIZE x {cal['write']:.3f}; "
          f"{steps} forwards)")
    print(f"{'kernel':44s} {'launches':>8s} {'read MB':>12s} {'written MB':>12s}")
    for k, n, rd, wr in rows:
        print(f"{k:44s} {n:8.2f} {rd / 1e6:12.1f} {wr / 1e6:12.1f}")
    print(f"{'all kernels of one forward':44s} {'':8s} {total / 1e6:12.1f} MB;  dominant kernel {dominant}: "
          f"{(dom[2] + dom[3]) / 1e6:.1f} MB")
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        rec = {}
    rec[workload + ("/prepared" if prepared else "")] = {
        "dominant_kernel": dominant, "dominant_kernel_bytes": int(dom[2] + dom[3]),
        "forward_bytes": int(total), "fetch_scale": cal["fetch"], "write_scale": cal["write"],
        "per_kernel": {k: {"launches": n, "read_bytes": int(rd), "written_bytes": int(wr)}
                       for k, n, rd, wr in rows}}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=15)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--path", default="auto", choices=["auto", "gather", "tile", "tile_split"])
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache launches")
    ap.add_argument("--suite", default=None, choices=["table3", "e2", "vf", "d128"],
                    help="instead of the benchmark line, time the shapes of the paper's Table III, "
                         "of its microbenchmark grid or of its model masks (Section V-F) and print one JSON object")
    ap.add_argument("--shapes", type=int, default=5, help="--suite d128: only the first N shapes (for a profile of one)")
    ap.add_argument("--dims", default="64,128,256",
                    help="head dimensions of --suite e2 (comma-separated)")
    ap.add_argument("--prepared", action="store_true",
                    help="explicit workloads: build the mask and prepare its tile graph once, "
                         "then time sga_attention_forward_prepared alone (the steady state that "
                         "the default line reports under steady_state)")
    ap.add_argument("--no-steady", action="store_true",
                    help="explicit workloads: skip the steady-state leg (prepared graph), so that a "
                         "profile of the run holds unprepared forwards only")
    ap.add_argument("--traffic-summary", default=None, metavar="DIR",
                    help="no GPU work: read the rocprofv3 --pmc csv files under DIR (see "
                         "traffic_summary) for --workload [--prepared], print the per-kernel HBM "
                         "bytes of one forward and record them in profiles/hbm_traffic.json")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain device copy of known size (1 GiB read + 1 GiB written) and "
                         "exit: the reference against which rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the hot path is a single-GPU kernel; "
              "no collectives exist). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.traffic_summary:
        traffic_summary(args.traffic_summary, args.workload, args.prepared)
        return
    import torch
    from sga_inputs import WORKLOADS, TABLE3_WORKLOADS, E2_RANDOM_WORKLOADS
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": n,
                          "bytes_written_per_copy": n, "copies": 5}))
        return
    path = {"auto": 0, "gather": 1, "tile": 2, "tile_split": 3}[args.path]
    if args.suite:
        print(json.dumps(suite_table3(path) if args.suite == "table3"
                         else suite_vf(path) if args.suite == "vf"
                         else suite_d128(path, args.shapes) if args.suite == "d128"
                         else suite_e2(path, tuple(int(x) for x in args.dims.split(",")))))
        return
    # (the long-context shapes of Table III can be named too, e.g. for a profile of one of them)
    wl = (WORKLOADS.get(args.workload) or TABLE3_WORKLOADS.get(args.workload)
          or E2_RANDOM_WORKLOADS[args.workload])
    run = Runner(wl, path)
    if args.prepared and wl.explicit:
        run.prepare()
    ms_step, fwd_ms, bld_ms, kern_ms = run.timed(args.steps, args.warmup)
    edges = run.nnz * wl.H
    step_name = ("sga_attention_forward_prepared (mask built and graph prepared once, outside the step)"
                 if run.prepared else "sga_build_mask + sga_attention_forward" if wl.explicit
                 else "sga_attention_forward_implicit")
    out = {
        "metric": "attention edges/s (q.k pairs)",
        "value": edges / (ms_step * 1e-3),
        "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "warmup_steps_run": run.warmup_steps_run,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "H": wl.H, "L": wl.L, "d": wl.d,
                   "mask": wl.mask.name, "explicit_csr": wl.explicit, "edges_per_step": edges,
                   "path": args.path, "seed": wl.seed, "step": step_name},
        "forward_ms": fwd_ms, "build_mask_ms": bld_ms,
        "forward_ms_min": run.min_forward_ms, "kernel_ms_min": run.min_kernel_ms,
        "ms_per_head": fwd_ms / wl.H,
        "forward_edges_per_s": edges / (fwd_ms * 1e-3),
        "roofline": roofline_of(wl, run.nnz, kern_ms, fwd_ms, args.path, run.kernel, run.prepared),
    }
    if not args.no_cold and fits_cache(wl):
        # one head's tensors fit the last-level cache: also report launches that start cold
        cf, ck = run.cold()
        out["cold_cache"] = {"forward_ms": cf, "kernel_ms": ck,
                             "how": "1 GiB scratch buffer overwritten before every launch, 5 launches"}
    if wl.explicit and not run.prepared and not args.no_steady:
        out["steady_state"] = steady_state(run, args.steps, args.warmup, args.path)
    if not args.no_cpu and not run.random:      # (the row-scan oracle takes mask predicates, not drawn CSR arrays)
        out["cpu_baseline"] = cpu_baseline(wl, run)
    del run
    torch.cuda.empty_cache()

    if not args.no_sweep:
        sweep = []
        # the five workloads, and the random CSR of the microbenchmark grid (Section V-C) that runs
        # on the per-row kernels
        general_csr = "e2_random_24k_sf0100_f32"
        for name, w in list(WORKLOADS.items()) + [(general_csr, E2_RANDOM_WORKLOADS[general_csr])]:
            if name == wl.name:
                continue
            try:
                r = Runner(w, path)
                if name == general_csr:
                    # no tile of this mask qualifies, and only a prepared graph knows that before
                    # the launch: its forward brackets the per-row kernel that does the work
                    r.prepare()
                ms, f, b, km = r.timed(20, 5)      # (each of these steps takes 0.05 to 2.5 ms)
                e = r.nnz * w.H
                sweep.append({"workload": name, "L": w.L, "H": w.H, "dtype": w.dtype, "prepared": r.prepared,
                              "edges_per_step": e, "ms_per_step": ms, "forward_ms": f,
                              "forward_ms_min": r.min_forward_ms, "kernel_ms_min": r.min_kernel_ms,
                              "build_mask_ms": b, "ms_per_head": f / w.H,
                              "forward_edges_per_s": e / (f * 1e-3),
                              "roofline": roofline_of(w, r.nnz, km, f, args.path, r.kernel, r.prepared)})
                if fits_cache(w):
                    cf, ck = r.cold()
                    sweep[-1]["cold_cache"] = {"forward_ms": cf, "kernel_ms": ck}
                if w.explicit and not r.prepared:
                    sweep[-1]["steady_state"] = steady_state(r, 20, 5, args.path)
                del r
            except Exception as ex:    # a sweep entry must not lose the headline line
                sweep.append({"workload": name, "error": repr(ex)})
            torch.cuda.empty_cache()
        out["sweep"] = sweep
        w2 = WORKLOADS["cfg2_longformer_64k"]
        if args.path == "auto":
            # workload 2 through the opt-in split-precision path (fp32 storage, three fp16
            # matrix-core products per product): reported beside the true-fp32 figures, never as them
            try:
                r = Runner(w2, 3)
                ms, f, b, km = r.timed(20, 5)
                out["split_precision"] = {"workload": w2.name, "path": "tile_split", "ms_per_step": ms,
                                          "forward_ms": f, "build_mask_ms": b,
                                          "forward_edges_per_s": r.nnz * w2.H / (f * 1e-3),
                                          "roofline": roofline_of(w2, r.nnz, km, f, "tile_split", r.kernel)}
                del r
            except Exception as ex:
                out["split_precision"] = {"error": repr(ex)}
            torch.cuda.empty_cache()
            try:
                out["composition"] = composition_times(w2, path, steps=20, warmup=5)
                # the same mask with fp16 storage (there the implicit pair is the faster one)
                import dataclasses
                out["composition_f16"] = composition_times(dataclasses.replace(w2, dtype="f16", sigma=0.5), path,
                                                           steps=20, warmup=5)
            except Exception as ex:
                out["composition"] = {"error": repr(ex)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
