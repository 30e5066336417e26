#!/usr/bin/env python3
"""Benchmark of the factorized-layer forward+backward path on one MI355X.

A step is one forward (T saved) plus one backward (dX, both factor gradients) of the
workload's factorized layer(s) on synthetic inputs that are already resident in HBM.  The
headline workload is the largest of the five benchmark configurations, the three
factorized convolutions of a ResNet-50 conv5_x bottleneck at batch 256 (bf16 inputs, fp32
accumulation); the other four configurations are measured in the same run and reported
in the `workloads` list of the same line.  Steps rotate over enough distinct buffer sets
to exceed the 256 MB last-level cache, so every step reads its activations from HBM.

Exactly --steps steps are timed per repetition (HIP-graph replay); repetitions are added
until at least 50 ms of GPU time have been measured, and the median repetition is reported
with the spread.

Prints ONE JSON line: throughput in algorithmic TFLOP/s (6 M r (C k^2 + Cout) per
factorized layer), the fraction of the MFMA peak and of min(peak, intensity x HBM
bandwidth), the roofline figures of the kernel that takes the most time (timed live with
HIP events around every launch), the dense un-factorized layer through the vendor
library, the same factorized layer as two vendor-library launches per direction with the
rank-r intermediate round-tripping HBM (the unfused leg), and the CPU oracle timed on
this machine's host cores, all cores and one.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "factorized-layer fwd+bwd TFLOP/s and % of MFMA peak vs dense layer, 1 MI355X"
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
HBM_GBS = 8000.0


# ----------------------------------------------------------------- workloads
class ConvWorkload:
    """One or more factorized convolutions (Section 2.2 shapes from Appendix D)."""

    def __init__(self, name, cfg):
        self.name, self.dtype = name, cfg["dtype"]
        if cfg["kind"] == "conv":
            self.layers = {"conv": (cfg["C"], cfg["Cout"], cfg["r"], cfg["k"], cfg["pad"])}
        else:
            self.layers = cfg["layers"]
        self.N, self.H, self.W, self.seed = cfg["N"], cfg["H"], cfg["W"], cfg["seed"]

    def describe(self):
        return {"workload": self.name, "batch": self.N, "hw": [self.H, self.W],
                "layers": {k: {"Cin": v[0], "Cout": v[1], "r": v[2], "k": v[3]} for k, v in self.layers.items()}}

    def flops(self):
        return sum(6.0 * self.N * self.H * self.W * r * (C * k * k + Co) for C, Co, r, k, p in self.layers.values())

    def dense_flops(self):
        return sum(6.0 * self.N * self.H * self.W * C * k * k * Co for C, Co, r, k, p in self.layers.values())

    def make_set(self, i, torch, workloads):
        sets = {}
        for lname, (C, Co, r, k, p) in self.layers.items():
            a = workloads.conv_inputs(self.N, C, self.H, self.W, Co, r, k, 1, p, dtype=self.dtype,
                                      seed=self.seed * 1000 + i)
            td = torch.bfloat16 if self.dtype == "bf16" else torch.float32
            sets[lname] = {n: torch.from_numpy(v).to(td).cuda().contiguous() for n, v in a.items()}
            sets[lname]["pad"] = p
        return sets

    def step(self, pf, s):
        for g in s.values():
            Y, T, Wsv = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], 1, g["pad"], save_T=True, save_W=True)
            pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], T_saved=T, stride=1, pad=g["pad"], W_saved=Wsv)

    def dense_prepare(self, s, torch):
        for g in s.values():
            if "Wd" not in g:
                g["Wd"] = torch.einsum("oq,qcij->ocij", g["Vp"].float(), g["Uk"].float()).to(g["X"].dtype).contiguous()

    def library_dense_prepare(self, s, torch):
        out = []
        for g in s.values():
            X = g["X"].detach().clone().requires_grad_(True)
            Wd = g["Wd"].detach().clone().requires_grad_(True)
            out.append((X, Wd, g["dY"], g["pad"]))
        return out

    def library_dense_step(self, prep, torch):
        for X, Wd, dY, pad in prep:
            X.grad = None
            Wd.grad = None
            torch.nn.functional.conv2d(X, Wd, padding=pad).backward(dY)

    def kernel_work(self):
        """{kernel name: [algorithmic flops per step, algorithmic bytes per step, launches per step]}, summed over
        the workload's layers (each layer launches each of its kernels once per step)."""
        s = 2 if self.dtype == "bf16" else 4
        out = {}

        def add(name, flops, nbytes):
            e = out.setdefault(name, [0.0, 0.0, 0])
            e[0] += flops
            e[1] += nbytes
            e[2] += 1

        for C, Co, r, k, p in self.layers.values():
            npix, K = self.N * self.H * self.W, C * k * k
            f1, f2 = 2.0 * npix * r * K, 2.0 * npix * r * Co  # one pass over the k x k stage / the 1x1 stage
            # any-shape path, one launch per contraction
            add("conv_T=Uk*X", f1, s * (npix * C + r * K + npix * r))
            add("conv_Y=Vp*T", f2, s * (npix * r + Co * r + npix * Co))
            add("conv_dT=Vpt*dY", f2, s * (npix * Co + Co * r) + 4 * npix * r)
            add("conv_dVp=dY*Tt", f2, s * (npix * Co + npix * r) + 4 * Co * r)
            add("conv_dX=Ukt*dT", f1, s * (r * K + npix * C) + 4 * npix * r)
            add("conv_dUk=dT*Xcolt", f1, s * npix * C + 4 * (npix * r + r * K))
            # fused small-image path
            add("conv_fwd_fused", f1 + f2, s * (npix * C + r * K + Co * r + npix * Co + npix * r))
            add("conv_bwd_data_fused", f1 + f2, s * (npix * Co + r * K + Co * r + npix * C + npix * r))
            add("conv_wgrad_pair", f1 + f2, s * (npix * C + npix * Co + 2 * npix * r) + 4 * (r * K + Co * r))
        return out

    def algorithmic_bytes(self):
        w = self.kernel_work()
        return sum(w[k][1] for k in ("conv_fwd_fused", "conv_bwd_data_fused", "conv_wgrad_pair"))

    def library_lowrank_prepare(self, s, torch):
        out = []
        for g in s.values():
            leaf = lambda t: t.detach().clone().requires_grad_(True)
            out.append((leaf(g["X"]), leaf(g["Uk"]), leaf(g["Vp"][:, :, None, None]), g["dY"], g["pad"]))
        return out

    def library_lowrank_step(self, prep, torch):
        """The factorized layer as the paper ran it: two library convolutions per direction, T through HBM."""
        F = torch.nn.functional
        for X, Uk, Vp, dY, pad in prep:
            X.grad = Uk.grad = Vp.grad = None
            F.conv2d(F.conv2d(X, Uk, padding=pad), Vp).backward(dY)

    def cpu_baseline(self, oracle, workloads, images=None):
        """Seconds of one fwd+bwd of every layer on `images` images of the batch (None = all), and its flops."""
        n = self.N if images is None else min(images, self.N)
        inputs = [(workloads.conv_inputs(n, C, self.H, self.W, Co, r, k, 1, p, dtype=self.dtype, seed=self.seed), p)
                  for C, Co, r, k, p in self.layers.values()]
        t0 = time.perf_counter()
        for a, p in inputs:
            oracle.lowrank_conv_fwd(a["X"], a["Uk"], a["Vp"], 1, p)
            oracle.lowrank_conv_bwd(a["X"], a["Uk"], a["Vp"], a["dY"], 1, p)
        secs = time.perf_counter() - t0
        return secs, self.flops() * n / self.N, f"fwd+bwd of every layer on {n} of {self.N} images, one run"

    def cpu_single_thread_sample(self):
        return max(1, self.N // 16)


class LinearWorkload:
    """One or more factorized linear layers (Section 2.1 / 2.4 shapes from Appendix D)."""

    def __init__(self, name, cfg):
        self.name, self.dtype, self.M, self.seed = name, cfg["dtype"], cfg["M"], cfg["seed"]
        self.layers = cfg["layers"] if cfg["kind"] == "linear_set" else {"fc": (cfg["n_in"], cfg["n_out"], cfg["r"])}
        # names of layers of one shape that read the same input and run through the shared-input entry points
        self.shared = tuple(cfg.get("shared", ()))

    def describe(self):
        d = {"workload": self.name, "tokens": self.M,
             "layers": {k: {"in": v[0], "out": v[1], "r": v[2]} for k, v in self.layers.items()}}
        if self.shared:
            d["shared_input"] = list(self.shared)
        return d

    def flops(self):
        return sum(6.0 * self.M * r * (i + o) for i, o, r in self.layers.values())

    def dense_flops(self):
        return sum(6.0 * self.M * i * o for i, o, r in self.layers.values())

    def make_set(self, idx, torch, workloads):
        td = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        out = {}
        for lname, (i, o, r) in self.layers.items():
            if lname in self.shared:
                continue
            a = workloads.linear_inputs(self.M, i, o, r, dtype=self.dtype, seed=self.seed * 1000 + idx, bias=True)
            out[lname] = {n: torch.from_numpy(v).to(td).cuda().contiguous() for n, v in a.items()}
        if self.shared:
            i, o, r = self.layers[self.shared[0]]
            a = workloads.linear_shared_inputs(self.M, i, o, r, len(self.shared), dtype=self.dtype,
                                               seed=self.seed * 1000 + idx, bias=True)
            out["+".join(self.shared)] = {n: torch.from_numpy(v).to(td).cuda().contiguous() for n, v in a.items()}
        return out

    def step(self, pf, s):
        for g in s.values():
            if g["V"].dim() == 3:
                Y, T = pf.pf_lowrank_linear_shared_fwd(g["X"], g["V"], g["U"], g["bias"], save_T=True)
                pf.pf_lowrank_linear_shared_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T, has_bias=True)
            else:
                Y, T = pf.pf_lowrank_linear_fwd(g["X"], g["V"], g["U"], g["bias"], save_T=True)
                pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T, has_bias=True)

    @staticmethod
    def _dense_layers(g):
        """(X, W, bias, dY) of every dense layer a set entry stands for."""
        if g["V"].dim() == 3:
            return [(g["X"], g["W"][k], g["bias"][k], g["dY"][k]) for k in range(g["V"].shape[0])]
        return [(g["X"], g["W"], g["bias"], g["dY"])]

    def dense_prepare(self, s, torch):
        for g in s.values():
            if "W" not in g:
                g["W"] = (g["U"].float() @ g["V"].float().transpose(-1, -2)).to(g["X"].dtype).contiguous()

    def library_dense_prepare(self, s, torch):
        out = []
        for g in s.values():
            for X, W, b, dY in self._dense_layers(g):
                out.append((X.detach().clone().requires_grad_(True), W.detach().clone().requires_grad_(True),
                            b.detach().clone().requires_grad_(True), dY))
        return out

    def library_dense_step(self, prep, torch):
        for X, W, b, dY in prep:
            X.grad = None
            W.grad = None
            b.grad = None
            torch.nn.functional.linear(X, W, b).backward(dY)

    def kernel_work(self):
        s = 2 if self.dtype == "bf16" else 4
        M = self.M
        out = {}

        def add(name, flops, nbytes):
            e = out.setdefault(name, [0.0, 0.0, 0])
            e[0] += flops
            e[1] += nbytes
            e[2] += 1

        for i, o, r in self.layers.values():
            add("linear_T=X*V", 2.0 * M * r * i, s * (M * i + i * r + M * r))
            add("linear_Y=T*Ut", 2.0 * M * r * o, s * (M * r + o * r + M * o))
            add("linear_dT=dY*U", 2.0 * M * r * o, s * (M * o + o * r) + 4 * M * r)
            add("linear_dX=dT*Vt", 2.0 * M * r * i, s * (i * r + M * i) + 4 * M * r)
            add("linear_dU=dYt*T", 2.0 * M * r * o, s * (M * o + M * r) + 4 * o * r)
            add("linear_dV=Xt*dT", 2.0 * M * r * i, s * M * i + 4 * (M * r + i * r))
            # fp32 with few rows: slices of the rank-r intermediate, then every product that reads their sum
            add("linear_T_slices", 2.0 * M * r * i, s * (M * i + i * r + M * r))
            add("linear_Y=T*Ut+b", 2.0 * M * r * o, s * (M * r + o * r + M * o + M * r))
            add("linear_dT_slices", 2.0 * M * r * o, s * (M * o + o * r + M * r))
            add("linear_dX,dU,dV,db", 2.0 * M * r * (2 * i + o), s * (2 * M * r + i * r + M * i + M * o + M * i) + 4 * r * (i + o))
            # fused path
            add("linear_fwd_fused", 2.0 * M * r * (i + o), s * (M * i + M * o + M * r + r * (i + o)))
            add("linear_bwd_data_fused", 2.0 * M * r * (i + o), s * (M * o + M * i + M * r + r * (i + o)))
            add("linear_wgrad_pair", 2.0 * M * r * (i + o), s * (M * i + M * o + 2 * M * r) + 4 * r * (i + o))
        if self.shared:  # one launch for all the projections of the shared input: X and dX move once
            i, o, r = self.layers[self.shared[0]]
            G = len(self.shared)
            add("linear_shared_fwd_fused", 2.0 * G * M * r * (i + o), s * (M * i + G * (M * o + M * r + r * (i + o))))
            add("linear_shared_bwd_data_fused", 2.0 * G * M * r * (i + o),
                s * (M * i + G * (M * o + M * r + r * (i + o))))
        return out

    def algorithmic_bytes(self):
        w = self.kernel_work()
        return sum(w[k][1] for k in ("linear_fwd_fused", "linear_bwd_data_fused", "linear_wgrad_pair"))

    def library_lowrank_prepare(self, s, torch):
        out = []
        leaf = lambda t: t.detach().clone().requires_grad_(True)
        for g in s.values():
            if g["V"].dim() == 3:
                for k in range(g["V"].shape[0]):
                    out.append((leaf(g["X"]), leaf(g["V"][k]), leaf(g["U"][k]), leaf(g["bias"][k]), g["dY"][k]))
            else:
                out.append((leaf(g["X"]), leaf(g["V"]), leaf(g["U"]), leaf(g["bias"]), g["dY"]))
        return out

    def library_lowrank_step(self, prep, torch):
        """The factorized layer as two library GEMMs per direction, T through HBM."""
        for X, V, U, b, dY in prep:
            X.grad = V.grad = U.grad = b.grad = None
            torch.nn.functional.linear(X @ V, U, b).backward(dY)

    def cpu_baseline(self, oracle, workloads, rows=None):
        """Seconds of one fwd+bwd of every layer on `rows` rows of the batch (None = all), and its flops."""
        m = self.M if rows is None else min(rows, self.M)
        inputs = [workloads.linear_inputs(m, i, o, r, dtype=self.dtype, seed=self.seed, bias=True)
                  for n, (i, o, r) in self.layers.items() if n not in self.shared]
        shared = None
        if self.shared:
            i, o, r = self.layers[self.shared[0]]
            shared = workloads.linear_shared_inputs(m, i, o, r, len(self.shared), dtype=self.dtype, seed=self.seed,
                                                    bias=True)
        t0 = time.perf_counter()
        for a in inputs:
            oracle.lowrank_linear_fwd(a["X"], a["V"], a["U"], a["bias"])
            oracle.lowrank_linear_bwd(a["X"], a["V"], a["U"], a["dY"])
        if shared:
            oracle.lowrank_linear_shared_fwd(shared["X"], shared["V"], shared["U"], shared["bias"])
            oracle.lowrank_linear_shared_bwd(shared["X"], shared["V"], shared["U"], shared["dY"])
        secs = time.perf_counter() - t0
        return secs, self.flops() * m / self.M, f"fwd+bwd of every layer on {m} of {self.M} rows, one run"

    def cpu_single_thread_sample(self):
        return max(1, self.M // 16)


class LstmWorkload:
    """The 2-layer factorized LSTM language model (Section 2.3, Appendix D): one step = forward through T time
    steps and back-propagation through time, one cell call per (time step, layer)."""

    def __init__(self, name, cfg, groups=1):
        self.name, self.dtype, self.cfg, self.groups = name, "f32", cfg, groups
        self.seq = bool(cfg.get("seq"))  # sequence-level entry points instead of one call per cell
        self.stack = bool(cfg.get("stack"))  # all layers in one call per direction

    def describe(self):
        c = self.cfg
        return {"workload": self.name, "seq_len": c["T"], "batch": c["B"], "layers": c["layers"], "d": c["d"],
                "h": c["h"], "r": c["r"], "groups": self.groups,
                "calls": "pf_lowrank_lstm_stack_*, one per direction" if self.stack else
                         "pf_lowrank_lstm_seq_*, one per layer and direction" if self.seq else
                         "pf_lowrank_lstm_cell_*, one per time step, layer and direction"}

    def flops(self):
        c = self.cfg
        per_cell = 6.0 * c["B"] * self.groups * c["r"] * (c["d"] + c["h"]) + 6.0 * c["B"] * c["r"] * 8 * c["h"]
        return per_cell * c["T"] * c["layers"]

    def dense_flops(self):
        c = self.cfg
        return 6.0 * c["B"] * 4 * c["h"] * (c["d"] + c["h"]) * c["T"] * c["layers"]

    def make_set(self, i, torch, workloads):
        c = self.cfg
        inp = workloads.lstm_lm_inputs(c["vocab"], c["d"], c["h"], c["r"], c["layers"], c["T"], c["B"],
                                       groups=self.groups, seed=c["seed"] * 1000 + i)
        g = {"x": torch.from_numpy(inp["E"][inp["tokens"]]).cuda().contiguous(),  # [T, B, d] embedded inputs
             "dH": torch.from_numpy(inp["dH_top"]).cuda().contiguous(),
             "P": [{k: torch.from_numpy(v).cuda().contiguous() for k, v in p.items()} for p in inp["layers"]],
             "zero": torch.zeros((c["B"], c["h"]), device="cuda")}
        return {"lm": g}

    def step_seq(self, pf, s):
        g = s["lm"]
        L, groups = len(g["P"]), self.groups
        x, saved = g["x"], []
        for p in g["P"]:
            out = pf.pf_lowrank_lstm_seq_fwd(x, g["zero"], g["zero"], p["Vx"], p["Ux"], p["Vh"], p["Uh"], p["bias"], groups)
            saved.append((x,) + out)
            x = out[0]
        above = g["dH"]
        for l in reversed(range(L)):
            p = g["P"][l]
            xin, h_all, c_all, gates_all, Tx_all, Th_all = saved[l]
            above, _, _, _ = pf.pf_lowrank_lstm_seq_bwd(xin, g["zero"], g["zero"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                        p["Vx"], p["Ux"], p["Vh"], p["Uh"], above, None, None, groups)

    def step_stack(self, pf, s):
        g = s["lm"]
        L, groups = len(g["P"]), self.groups
        col = lambda k: [p[k] for p in g["P"]]
        zero = [g["zero"]] * L
        Vx, Ux, Vh, Uh = col("Vx"), col("Ux"), col("Vh"), col("Uh")
        saved = pf.pf_lowrank_lstm_stack_fwd(g["x"], zero, zero, Vx, Ux, Vh, Uh, col("bias"), groups)
        pf.pf_lowrank_lstm_stack_bwd(g["x"], zero, zero, *saved, Vx, Ux, Vh, Uh, g["dH"], None, None, groups)

    def step(self, pf, s):
        if self.stack:
            return self.step_stack(pf, s)
        if self.seq:
            return self.step_seq(pf, s)
        g = s["lm"]
        T, L, groups = g["x"].shape[0], len(g["P"]), self.groups
        hs, cs = [g["zero"]] * L, [g["zero"]] * L
        saved = [[None] * T for _ in range(L)]
        for t in range(T):
            x = g["x"][t]
            for l, p in enumerate(g["P"]):
                ho, co, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(x, hs[l], cs[l], p["Vx"], p["Ux"], p["Vh"], p["Uh"],
                                                                    p["bias"], groups)
                saved[l][t] = (x, hs[l], cs[l], co, gates, Tx, Th)
                hs[l], cs[l] = ho, co
                x = ho
        grads = [None] * L
        dh_next, dc_next = [g["zero"]] * L, [g["zero"]] * L
        for t in reversed(range(T)):
            above = g["dH"][t]
            for l in reversed(range(L)):
                p = g["P"][l]
                x, hp, cp, co, gates, Tx, Th = saved[l][t]
                dx, dhp, dcp, grads[l] = pf.pf_lowrank_lstm_cell_bwd(x, hp, cp, co, gates, Tx, Th, p["Vx"], p["Ux"],
                                                                     p["Vh"], p["Uh"], above + dh_next[l], dc_next[l],
                                                                     groups, grads=grads[l])
                dh_next[l], dc_next[l] = dhp, dcp
                above = dx

    def kernel_work(self):
        """Small-batch path: five contraction/update launches per cell; algorithmic bytes count every factor once per
        launch that uses it, activations once, and the accumulated gradients as read + write."""
        c = self.cfg
        B, d, h, r, g = c["B"], c["d"], c["h"], c["r"], self.groups
        gr, cells = g * r, c["T"] * c["layers"]
        if self.stack or self.seq:
            # one call per direction for the whole stack, or (sequence entry points) per layer: a slot holds every
            # layer of the call that has a step on its diagonal
            Mt, L = c["T"] * B, c["layers"]
            calls, lay = (1, L) if self.stack else (L, 1)
            slots = calls * (c["T"] + lay - 1)
            up = (lay - 1) * c["T"] * calls  # layer-to-layer products that ride in the slots
            prods = cells + up
            ws = {
                "lstm_stack_T": (2.0 * B * gr * h * prods, 4 * (gr * h + B * h + B * gr) * prods, slots),
                "lstm_stack_z": (2.0 * B * 4 * h * r * prods, 4 * (4 * h * r + B * gr + 2 * B * 4 * h) * prods, slots),
                # pre-activations of both paths and the gates in one launch (one factor pair per path)
                "lstm_stack_z_gates": (2.0 * B * 4 * h * r * 2 * cells,
                                       4 * ((4 * h * r + B * gr) * 2 * cells + (B * 4 * h + 3 * B * h) * cells), slots),
                "lstm_stack_dT": (2.0 * B * 4 * h * r * prods, 4 * (4 * h * r + B * 4 * h + B * gr) * prods, slots),
                "lstm_stack_dh": (2.0 * B * gr * h * prods, 4 * (gr * h + B * gr + B * h) * prods, slots),
                # dh from both products and the gate derivatives in one launch (one factor pair per path)
                "lstm_stack_dh_gates": (2.0 * B * gr * h * prods,
                                        4 * ((gr * h + B * gr) * prods + (B * 4 * h * 2 + 5 * B * h) * cells),
                                        slots + calls),
                "lstm_stack_grads": (2.0 * Mt * (8 * h * r + gr * (d + h)) * L,
                                     4 * ((8 * h * r + gr * (d + h) + 4 * h) + Mt * (4 * h + 2 * gr + d + h)) * L,
                                     L if Mt >= 128 else 2 * L),  # one launch per layer from 128 rows on
            }
            return {k: [f, b, n] for k, (f, b, n) in ws.items()}
        w = {
            "lstm_T=[x*Vx|h*Vh]": (2.0 * B * gr * (d + h), 4 * (gr * (d + h) + B * (d + h) + 2 * B * gr)),
            "lstm_z=[Tx|Th]*[Ux|Uh]t": (2.0 * B * 4 * h * 2 * r, 4 * (8 * h * r + 2 * B * gr + B * 4 * h)),
            "lstm_dT=dz*[Ux|Uh]": (2.0 * B * 4 * h * 2 * r, 4 * (8 * h * r + B * 4 * h + 2 * B * gr)),
            "lstm_dxh=[dTx*Vxt|dTh*Vht]": (2.0 * B * gr * (d + h), 4 * (gr * (d + h) + 2 * B * gr + B * (d + h))),
            "lstm_grads": (2.0 * B * (8 * h * r + gr * (d + h)),
                           4 * (2 * (8 * h * r + gr * (d + h) + 4 * h) + B * (4 * h + 2 * gr + d + h))),
        }
        return {k: [f * cells, b * cells, cells] for k, (f, b) in w.items()}

    def algorithmic_bytes(self):
        w = self.kernel_work()
        if self.stack or self.seq:
            names = (("lstm_stack_T", "lstm_stack_z_gates", "lstm_stack_dT", "lstm_stack_dh_gates", "lstm_stack_grads")
                     if self.groups == 1 else ("lstm_stack_T", "lstm_stack_z", "lstm_stack_dT", "lstm_stack_dh", "lstm_stack_grads"))
            return sum(w[k][1] for k in names)
        return sum(v[1] for v in w.values())

    def cpu_baseline(self, oracle, workloads, cells=8):
        """Seconds of `cells` cell steps (fwd+bwd) of one layer, and their flops."""
        c = self.cfg
        n = cells or 8
        a = workloads.lstm_cell_inputs(c["B"], c["d"], c["h"], c["r"], groups=self.groups, seed=c["seed"])
        t0 = time.perf_counter()
        for _ in range(n):
            ho, co, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(a["x"], a["h_prev"], a["c_prev"], a["Vx"], a["Ux"],
                                                                 a["Vh"], a["Uh"], a["bias"], self.groups)
            oracle.lowrank_lstm_cell_bwd(a["x"], a["h_prev"], a["c_prev"], co, gates, Tx, Th, a["Vx"], a["Ux"], a["Vh"],
                                         a["Uh"], a["dh"], a["dc"], self.groups)
        secs = time.perf_counter() - t0
        return secs, self.flops() / (c["T"] * c["layers"]) * n, \
            f"{n} cell steps (fwd+bwd) of one layer; the full workload is {c['T'] * c['layers']} of them"

    def cpu_single_thread_sample(self):
        return 2


class FfnBlockWorkload:
    """y = x + FFN(x), FFN(x) = max(0, x W1 + b1) W2 + b2 (Section 2.4) with both matrices factorized: two
    pf_lowrank_linear_fwd_ep calls forward, two pf_lowrank_linear_bwd_ep calls backward (the ReLU mask applied where
    dH is formed, the skip gradient where dx is formed)."""

    def __init__(self, name, cfg):
        self.name, self.dtype, self.cfg = name, cfg["dtype"], cfg
        c = cfg
        self.inner = LinearWorkload(name, dict(kind="linear_set", dtype=c["dtype"], M=c["M"], seed=c["seed"], layers=dict(
            ffn1=(c["d"], c["dff"], c["r"]), ffn2=(c["dff"], c["d"], c["r"]))))

    def describe(self):
        c = self.cfg
        return {"workload": self.name, "tokens": c["M"], "d_model": c["d"], "d_ff": c["dff"], "r": c["r"],
                "calls": "pf_lowrank_linear_fwd_ep / pf_lowrank_linear_bwd_ep"}

    def flops(self):
        return self.inner.flops()

    def dense_flops(self):
        return self.inner.dense_flops()

    def algorithmic_bytes(self):
        return self.inner.algorithmic_bytes()

    def kernel_work(self):
        return self.inner.kernel_work()

    def make_set(self, i, torch, workloads):
        return self.inner.make_set(i, torch, workloads)

    def step(self, pf, s):
        g1, g2 = s["ffn1"], s["ffn2"]
        H, T1 = pf.pf_lowrank_linear_fwd_ep(g1["X"], g1["V"], g1["U"], g1["bias"], act="relu")
        Y, T2 = pf.pf_lowrank_linear_fwd_ep(H, g2["V"], g2["U"], g2["bias"], residual=g1["X"])
        dZ1, _, _, _ = pf.pf_lowrank_linear_bwd_ep(H, g2["V"], g2["U"], g2["dY"], T_saved=T2, x_is_relu=True, has_bias=True)
        pf.pf_lowrank_linear_bwd_ep(g1["X"], g1["V"], g1["U"], dZ1, T_saved=T1, dX_add=g2["dY"], has_bias=True)

    def separate_step(self, pf, s, torch):
        """The same block with the plain calls and the element-wise steps as separate (torch) kernels."""
        g1, g2 = s["ffn1"], s["ffn2"]
        H, T1 = pf.pf_lowrank_linear_fwd(g1["X"], g1["V"], g1["U"], g1["bias"])
        H = torch.relu_(H)
        Y, T2 = pf.pf_lowrank_linear_fwd(H, g2["V"], g2["U"], g2["bias"])
        Y += g1["X"]
        dH, _, _, _ = pf.pf_lowrank_linear_bwd(H, g2["V"], g2["U"], g2["dY"], T_saved=T2, has_bias=True)
        dH *= (H > 0)
        dx, _, _, _ = pf.pf_lowrank_linear_bwd(g1["X"], g1["V"], g1["U"], dH, T_saved=T1, has_bias=True)
        dx += g2["dY"]

    def cpu_baseline(self, oracle, workloads, rows=None):
        return self.inner.cpu_baseline(oracle, workloads, rows)

    def cpu_single_thread_sample(self):
        return self.inner.cpu_single_thread_sample()


class BasicBlockWorkload:
    """A ResNet-18 basic block (Appendix D) of two factorized 3x3 convolutions, batch norm with fixed statistics and
    ReLU after each, identity shortcut: y1 = relu(bn1(conv1(x))), y2 = relu(bn2(conv2(y1)) + x), through
    pf_lowrank_conv_fwd_ep / pf_lowrank_conv_bwd_ep."""

    def __init__(self, name, cfg):
        self.name, self.dtype, self.cfg = name, cfg["dtype"], cfg
        c = cfg
        self.inner = ConvWorkload(name, dict(kind="conv_set", dtype=c["dtype"], N=c["N"], H=c["H"], W=c["W"], seed=c["seed"],
                                             layers=dict(conv1=(c["C"], c["C"], c["r"], c["k"], c["k"] // 2),
                                                         conv2=(c["C"], c["C"], c["r"], c["k"], c["k"] // 2))))

    def describe(self):
        d = self.inner.describe()
        d["calls"] = "pf_lowrank_conv_fwd_ep / pf_lowrank_conv_bwd_ep"
        return d

    def flops(self):
        return self.inner.flops()

    def dense_flops(self):
        return self.inner.dense_flops()

    def algorithmic_bytes(self):
        return self.inner.algorithmic_bytes()

    def kernel_work(self):
        return self.inner.kernel_work()

    def make_set(self, i, torch, workloads):
        s = self.inner.make_set(i, torch, workloads)
        C = self.cfg["C"]
        for j, g in enumerate(s.values()):
            gen = torch.Generator(device="cpu").manual_seed(1000 * i + j)
            g["scale"] = (0.5 + torch.rand(C, generator=gen)).cuda()
            g["shift"] = (0.2 * torch.randn(C, generator=gen)).cuda()
        s["conv1"]["X"] = torch.relu(s["conv1"]["X"])
        return s

    def step(self, pf, s):
        g1, g2 = s["conv1"], s["conv2"]
        p = g1["pad"]
        y1, T1, W1 = pf.pf_lowrank_conv_fwd_ep(g1["X"], g1["Uk"], g1["Vp"], g1["scale"], g1["shift"], act="relu", stride=1,
                                               pad=p, save_W=True)
        y2, T2, W2 = pf.pf_lowrank_conv_fwd_ep(y1, g2["Uk"], g2["Vp"], g2["scale"], g2["shift"], residual=g1["X"], act="relu",
                                               stride=1, pad=p, save_W=True)
        dZ2 = g2["dY"]  # (what the block above hands down)
        dZ1, _, _, _ = pf.pf_lowrank_conv_bwd_ep(y1, g2["Uk"], g2["Vp"], g2["scale"], dZ2, T_saved=T2, stride=1, pad=p,
                                                 x_is_relu=True, W_saved=W2)
        pf.pf_lowrank_conv_bwd_ep(g1["X"], g1["Uk"], g1["Vp"], g1["scale"], dZ1, T_saved=T1, stride=1, pad=p, dX_add=dZ2,
                                  x_is_relu=True, W_saved=W1)

    def separate_step(self, pf, s, torch):
        g1, g2 = s["conv1"], s["conv2"]
        p = g1["pad"]
        bn = lambda y, g: y.mul_(g["scale"].to(y.dtype)[None, :, None, None]).add_(g["shift"].to(y.dtype)[None, :, None, None])
        y1, T1, W1 = pf.pf_lowrank_conv_fwd(g1["X"], g1["Uk"], g1["Vp"], 1, p, save_W=True)
        y1 = torch.relu_(bn(y1, g1))
        y2, T2, W2 = pf.pf_lowrank_conv_fwd(y1, g2["Uk"], g2["Vp"], 1, p, save_W=True)
        y2 = torch.relu_(bn(y2, g2).add_(g1["X"]))
        dZ2 = g2["dY"]
        dP2 = dZ2 * g2["scale"].to(dZ2.dtype)[None, :, None, None]
        dsh2 = dZ2.float().sum(dim=(0, 2, 3))
        dy1, _, _ = pf.pf_lowrank_conv_bwd(y1, g2["Uk"], g2["Vp"], dP2, T_saved=T2, stride=1, pad=p, W_saved=W2)
        dy1 *= (y1 > 0)
        dP1 = dy1 * g1["scale"].to(dy1.dtype)[None, :, None, None]
        dsh1 = dy1.float().sum(dim=(0, 2, 3))
        dx, _, _ = pf.pf_lowrank_conv_bwd(g1["X"], g1["Uk"], g1["Vp"], dP1, T_saved=T1, stride=1, pad=p, W_saved=W1)
        dx += dZ2
        dx *= (g1["X"] > 0)

    def cpu_baseline(self, oracle, workloads, images=None):
        return self.inner.cpu_baseline(oracle, workloads, images)

    def cpu_single_thread_sample(self):
        return self.inner.cpu_single_thread_sample()


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None when there is no
    figure or the kernel's source file has changed since the counters were taken."""
    import glob
    import hashlib
    for path in glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic.md")):
        for line in open(path):
            f = line.split()
            if len(f) == 6 and f[0] == "traffic" and f[1] == workload and f[2] == kernel:
                src = os.path.join(ROOT, f[4])
                if os.path.exists(src) and hashlib.sha256(open(src, "rb").read()).hexdigest() == f[5]:
                    return float(f[3])
    return None


def svd_bench(args, torch, pf, workloads):
    """Truncated-SVD factor initialisation (Algorithm 1), not part of the training step: one line with the time per
    matrix on the GPU and, for the smallest matrix, the oracle's time on the host."""
    cfg = workloads.CONFIGS[args.workload]
    res = {}
    for name, (m, n, r) in cfg["layers"].items():
        W = torch.from_numpy(workloads.Stream(workloads.SEED_BASE + cfg["seed"], "f32").normal((m, n)).astype("float32")).cuda()
        pf.pf_svd_split(W, r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = max(1, min(args.steps, 3))
        for _ in range(reps):
            pf.pf_svd_split(W, r)
        torch.cuda.synchronize()
        res[name] = {"m": m, "n": n, "r": r, "ms": (time.perf_counter() - t0) / reps * 1e3}
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        name, (m, n, r) = next(iter(cfg["layers"].items()))
        W = workloads.Stream(workloads.SEED_BASE + cfg["seed"], "f32").normal((m, n))
        t0 = time.perf_counter()
        oracle.svd_split(W, r)
        cpu = {"value": 1.0 / (time.perf_counter() - t0), "unit": "factorizations/s", "cores": 1, "kind": "oracle",
               "sample": f"{name} ({m} x {n}, r = {r}) only"}
    total_ms = sum(v["ms"] for v in res.values())
    print(json.dumps({
        "metric": "truncated-SVD factor initialisation (Algorithm 1), layer matrices factorized per second, 1 MI355X",
        "value": len(res) / (total_ms * 1e-3), "unit": "factorizations/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": total_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic", "config": {"workload": args.workload, "layers": res}, "roofline": None,
        "cpu_baseline": cpu}))


def make_workload(name, lstm_groups=1):
    import workloads
    cfg = workloads.CONFIGS[name]
    if cfg["kind"] in ("conv", "conv_set"):
        return ConvWorkload(name, cfg)
    if cfg["kind"] in ("linear", "linear_set"):
        return LinearWorkload(name, cfg)
    if cfg["kind"] == "lstm":
        return LstmWorkload(name, cfg, groups=lstm_groups)
    if cfg["kind"] == "ffn_block":
        return FfnBlockWorkload(name, cfg)
    if cfg["kind"] == "basic_block":
        return BasicBlockWorkload(name, cfg)
    raise SystemExit(f"unknown workload {name}")


MIN_TIMED_MS = 50.0   # GPU time measured per figure, at least
MAX_REPEATS = 400


def _repeat(torch, run_once, steps):
    """Times run_once() (exactly `steps` steps) again and again until MIN_TIMED_MS of GPU time are on record; returns
    the ms/step of every repetition."""
    per_rep, total = [], 0.0
    while (total < MIN_TIMED_MS or len(per_rep) < 3) and len(per_rep) < MAX_REPEATS:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run_once()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        per_rep.append(ms / steps)
        total += ms
    return per_rep


def time_steps(torch, fn, sets, steps, warmup):
    """Eager launches: `warmup` untimed steps, then repetitions of exactly `steps` timed steps."""
    for i in range(warmup):
        fn(sets[i % len(sets)])
    torch.cuda.synchronize()

    def once():
        for i in range(steps):
            fn(sets[i % len(sets)])
    return _repeat(torch, once, steps)


def capture_graph(torch, fn, sets, count):
    """One HIP graph holding `count` whole steps (all launches of fwd + bwd), walking the buffer sets in turn."""
    for s in sets:
        fn(s)  # eager once: output tensors of the right size are in torch's pool before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(count):
            fn(sets[i % len(sets)])
    return g


def time_graph_steps(torch, fn, sets, steps, warmup):
    """Exactly `steps` steps per repetition, as replays of one graph of len(sets) steps plus one graph for the
    remainder."""
    per = len(sets)
    full = capture_graph(torch, fn, sets, per) if steps >= per else None
    rem = capture_graph(torch, fn, sets, steps % per) if steps % per else None
    for i in range(max(1, warmup // per)):
        (full or rem).replay()
    torch.cuda.synchronize()

    def once():
        for i in range(steps // per):
            full.replay()
        if rem is not None:
            rem.replay()
    return _repeat(torch, once, steps)


def summary(per_rep):
    return {"ms_per_step": statistics.median(per_rep), "repeats": len(per_rep), "min_ms_per_step": min(per_rep),
            "max_ms_per_step": max(per_rep)}


def host_description():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "cpu_model": model}


def cpu_baseline(wl, workloads):
    """The oracle on this machine's host cores: all threads on (a bounded sample of) the workload, then one thread
    on a smaller sample of it."""
    import oracle
    threads = oracle.num_threads()
    secs, cflops, sample = wl.cpu_baseline(oracle, workloads)
    out = {"value": cflops / secs / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle", "sample": sample,
           "seconds": secs}
    oracle.set_num_threads(1)
    try:
        s1, f1, sample1 = wl.cpu_baseline(oracle, workloads, wl.cpu_single_thread_sample())
    finally:
        oracle.set_num_threads(threads)
    out["single_thread"] = {"value": f1 / s1 / 1e12, "unit": "TFLOP/s", "cores": 1, "sample": sample1, "seconds": s1}
    out.update(host_description())
    return out


def run_workload(args, torch, pf, workloads, name, lstm_groups=1):
    """Every figure of one workload, as a dict."""
    wl = make_workload(name, lstm_groups)
    one = wl.make_set(0, torch, workloads)
    set_bytes = sum(t.numel() * t.element_size() for g in one.values() for t in g.values() if hasattr(t, "numel"))
    nsets = args.buffer_sets or max(2, int(300e6 // max(set_bytes * 2, 1)) + 1)  # x2: outputs are as large as inputs
    nsets = min(nsets, 64)
    sets = [one] + [wl.make_set(i, torch, workloads) for i in range(1, nsets)]
    step = lambda s: wl.step(pf, s)

    eager = summary(time_steps(torch, step, sets, args.steps, args.warmup))
    if args.no_graph:
        timed = eager
        resident = summary(time_steps(torch, step, sets[:1], args.steps, args.warmup))
    else:
        # a step is a handful of microsecond kernels, launch-bound from the host, so it is replayed as a HIP graph
        timed = summary(time_graph_steps(torch, step, sets, args.steps, args.warmup))
        resident = summary(time_graph_steps(torch, step, sets[:1] * 8, args.steps, args.warmup))
    ms = timed["ms_per_step"]
    flops = wl.flops()
    value = flops / (ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[wl.dtype]
    ai = flops / wl.algorithmic_bytes()
    attainable = min(peak, ai * HBM_GBS / 1e3)  # TFLOP/s: min(MFMA peak, intensity x HBM bandwidth)

    # per-kernel durations, HIP events around every launch on the launch stream
    pf.timing_reset()
    pf.timing_enable(True)
    for i in range(max(args.steps, 20)):
        wl.step(pf, sets[i % len(sets)])
    torch.cuda.synchronize()
    pf.timing_enable(False)
    per_kernel = pf.timing_collect()
    kernels = {k: {"launches": n, "avg_us": 1e3 * t / n} for k, (n, t) in sorted(per_kernel.items(), key=lambda kv: -kv[1][1])}
    work = wl.kernel_work()
    roofline = None
    if kernels:
        dom = next((k for k in kernels if k in work), next(iter(kernels)))  # the costliest kernel that has a work model
        roofline = {"kernel": dom, "bound": "mfma", "achieved": None, "peak": peak, "unit": "TFLOP/s", "frac": None,
                    "traffic": None, "avg_us": kernels[dom]["avg_us"]}
        if dom in work:
            kflops, kbytes, per_step = work[dom]
            step_s = kernels[dom]["avg_us"] * 1e-6 * per_step  # time this kernel takes per step, all layers
            bound = "mfma" if kflops / kbytes >= peak * 1e12 / (HBM_GBS * 1e9) else "hbm"
            roofline.update({"bound": bound, "launches_per_step": per_step, "algorithmic_flops_per_step": kflops,
                             "algorithmic_bytes_per_step": kbytes, "traffic": measured_traffic(wl.name, dom)})
            if bound == "mfma":
                roofline.update({"achieved": kflops / step_s / 1e12, "peak": peak, "unit": "TFLOP/s",
                                 "frac": kflops / step_s / 1e12 / peak})
            else:
                roofline.update({"achieved": kbytes / step_s / 1e9, "peak": HBM_GBS, "unit": "GB/s",
                                 "frac": kbytes / step_s / 1e9 / HBM_GBS})
            roofline["tflops"] = kflops / step_s / 1e12
            roofline["algorithmic_GBps"] = kbytes / step_s / 1e9

    def vendor_leg(prepare, run):
        """ms/step summary of a torch (vendor library) leg: graph-replayed like the factorized path when torch can
        capture it, else launched eagerly."""
        prep = [prepare(s_, torch) for s_ in sets[:4]]
        fn = lambda p: run(p, torch)
        if not args.no_graph:
            try:
                return dict(summary(time_graph_steps(torch, fn, prep, args.steps, 4)), launch="hip_graph")
            except Exception:
                torch.cuda.synchronize()
        return dict(summary(time_steps(torch, fn, prep, args.steps, 5)), launch="eager")

    library = unfused = None
    if not args.no_dense and hasattr(wl, "library_dense_step"):
        # the dense layer through the vendor library (torch -> MIOpen / hipBLASLt), as an outside reference
        try:
            for s_ in sets[:4]:
                wl.dense_prepare(s_, torch)
            lms = vendor_leg(wl.library_dense_prepare, wl.library_dense_step)
            library = dict(lms, value=wl.dense_flops() / (lms["ms_per_step"] * 1e-3) / 1e12, unit="TFLOP/s (dense flops)",
                           what=f"torch.nn.functional dense layer fwd+bwd, {wl.dtype}, vendor library kernels",
                           speedup_of_factorized=lms["ms_per_step"] / ms)
        except Exception as e:  # the outside reference is optional
            library = {"error": repr(e)[:200]}
        # the factorized layer as two library launches per direction: the rank-r intermediate goes through HBM
        try:
            ums = vendor_leg(wl.library_lowrank_prepare, wl.library_lowrank_step)
            unfused = dict(ums, value=flops / (ums["ms_per_step"] * 1e-3) / 1e12, unit="TFLOP/s",
                           what="the same factorized layer as two vendor-library launches per direction (torch autograd), "
                                "T written to and read back from HBM",
                           speedup_of_fused=ums["ms_per_step"] / ms)
        except Exception as e:
            unfused = {"error": repr(e)[:200]}

    separate = None
    if hasattr(wl, "separate_step"):
        sep = lambda s_: wl.separate_step(pf, s_, torch)
        sms = summary(time_steps(torch, sep, sets, args.steps, args.warmup) if args.no_graph else
                      time_graph_steps(torch, sep, sets, args.steps, args.warmup))
        separate = dict(sms, what="the same block through the plain calls, its element-wise steps as separate kernels",
                        speedup_of_fused_epilogues=sms["ms_per_step"] / ms)

    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, workloads)
    del sets, one
    torch.cuda.empty_cache()
    return {
        "value": value, "unit": "TFLOP/s", "ms_per_step": ms, "dtype": wl.dtype,
        "config": dict(wl.describe(), buffer_sets=nsets),
        "timing": timed, "frac_of_mfma_peak": value / peak,
        "arithmetic_intensity": ai, "attainable_TFLOPs": attainable, "frac_of_min_peak_ai_bw": value / attainable,
        "launch": "eager" if args.no_graph else "hip_graph", "eager_ms_per_step": eager["ms_per_step"],
        "cache_resident": {"ms_per_step": resident["ms_per_step"], "value": flops / (resident["ms_per_step"] * 1e-3) / 1e12},
        "roofline": roofline, "cpu_baseline": cpu, "dense_layer_vendor_library": library,
        "unfused_vendor_library": unfused, "separate_epilogues": separate, "kernels": kernels,
    }


# the five benchmark configurations, largest first (the first is the headline unless --workload names another)
FIVE = ["resnet50_conv5_bf16", "transformer_block_bf16", "lstm_lm_stack_f32", "resnet18_conv4_bf16", "linear_fc_f32"]
# two blocks that run the layers with their epilogues (not among the five configurations; reported after them)
BLOCKS = ["transformer_ffn_block_bf16", "resnet18_basic_block_bf16"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=FIVE[0])
    ap.add_argument("--single", action="store_true", help="measure --workload only, not the other four configurations")
    ap.add_argument("--buffer-sets", type=int, default=0, help="distinct input/output sets to rotate over (0 = enough to exceed 256 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the vendor-library legs (dense layer, unfused factorized layer)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy, so that byte counters of a profiler run can be scaled")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of replaying HIP graphs")
    ap.add_argument("--lstm-groups", type=int, default=1, choices=(1, 4),
                    help="LSTM workloads: 1 = one factor pair per path, 4 = one pair per gate and path (Appendix D's table)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import torch
    import workloads
    import paper_2103_03936_amd as pf

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: the HIP library has no CPU path")
    torch.cuda.set_device(0)
    if workloads.CONFIGS[args.workload]["kind"] == "svd":
        return svd_bench(args, torch, pf, workloads)

    head = run_workload(args, torch, pf, workloads, args.workload, args.lstm_groups)
    others = []
    if not args.single:
        for name in FIVE:
            if name == args.workload:
                continue
            r = run_workload(args, torch, pf, workloads, name, 1)
            others.append(r)
            if workloads.CONFIGS[name]["kind"] == "lstm":  # the paper's own reading: one factor pair per gate and path
                others.append(run_workload(args, torch, pf, workloads, name, 4))
        saved, args.no_dense, args.no_cpu_baseline = (args.no_dense, args.no_cpu_baseline), True, True
        for name in BLOCKS:
            if name != args.workload:
                others.append(run_workload(args, torch, pf, workloads, name, 1))
        args.no_dense, args.no_cpu_baseline = saved

    if args.copy_calibration:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()

    out = {
        "metric": METRIC, "value": head["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
    }
    out.update({k: v for k, v in head.items() if k not in out})
    brief = lambda r: {k: r[k] for k in ("config", "dtype", "ms_per_step", "value", "unit", "timing", "frac_of_mfma_peak",
                                         "arithmetic_intensity", "attainable_TFLOPs", "frac_of_min_peak_ai_bw",
                                         "eager_ms_per_step", "roofline", "cpu_baseline", "dense_layer_vendor_library",
                                         "unfused_vendor_library", "separate_epilogues", "kernels")}
    out["workloads"] = [brief(head)] + [brief(r) for r in others]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
