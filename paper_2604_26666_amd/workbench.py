"""The benchmark configurations as runnable cases, for bench.py --all and the on-device sweep.

Each case names one GEMM of the five configurations (shapes from the workload definition;
see workloads/__init__.py), allocates its seeded inputs on the GPU and launches it through
the C ABI.  PyTorch is used for device memory and event timing only.
"""
import torch

from . import binding as fact

PEAK_BF16_TFLOPS = 2516.6
PEAK_HBM_GBS = 8000.0


class Case:
    def __init__(self, name, M, N, K, trans_b, act=fact.ACT_NONE, bias=False, residual=False, batch=1,
                 splitk=False, maker=None):
        self.name, self.M, self.N, self.K, self.trans_b, self.act = name, M, N, K, trans_b, act
        self.has_bias, self.has_res, self.batch, self.splitk = bias, residual, batch, splitk
        self.maker = maker
        self.t = None

    @property
    def nout(self):
        return self.N // 2 if self.act == fact.ACT_SILU_GATE else self.N

    @property
    def flops(self):
        return 2.0 * self.M * self.N * self.K * self.batch

    @property
    def min_bytes(self):
        b = self.batch * (self.M * self.K + self.K * self.N + self.M * self.nout) * 2.0
        if self.has_bias:
            b += self.nout * 2.0
        if self.has_res:
            b += self.batch * self.M * self.nout * 2.0
        return b

    def alloc(self):
        if self.t is None:
            t = {k: (v.cuda() if v is not None else None) for k, v in self.maker().items()}
            shape = (self.batch, self.M, self.nout) if self.batch > 1 else (self.M, self.nout)
            t["C"] = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
            t["ws"] = None
            self.t = t
        return self.t

    def free(self):
        self.t = None

    def _ws(self, nbytes):
        t = self.t
        if nbytes > 0 and (t["ws"] is None or t["ws"].numel() < nbytes):
            t["ws"] = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        return t["ws"]

    def run(self, cfg=-1, split=0, group_m=0):
        """Launch once.  cfg/split/group_m <= 0 (split 0) leave the choice to the table.  Returns the status."""
        t = self.alloc()
        ep = fact.Epilogue(bias=t.get("bias"), residual=t.get("R"), ldr=self.nout,
                           stride_r=self.M * self.nout if self.batch > 1 else 0, act=self.act)
        lda = self.K
        ldb = self.K if self.trans_b else self.N
        if self.batch > 1 and split == 0:
            split = 1
        # split 0 = the table's choice, which may be a split-K or a tail split: both need a workspace
        need = fact.fact_gemm_splitk_workspace_bytes(self.M, self.N, self.K, split) if split != 1 else 0
        ws = self._ws(need)
        return fact.fact_gemm_ex(self.batch, self.M, self.N, self.K, t["A"], lda, self.M * self.K,
                                 t["B"], ldb, self.K * self.N, self.trans_b, t["C"], self.nout, self.M * self.nout,
                                 ep, cfg, split, group_m, ws, need)


def cases(names=None):
    import workloads as wl

    def c1():
        c = wl.config1()
        return {"A": c["A"], "B": c["B"]}

    def c2():
        c = wl.config2()
        return {"A": c["A"], "B": c["B"], "bias": c["bias"]}

    def c3a():
        c = wl.config3a()
        return {"A": c["A"], "B": c["B"]}

    def c3b():
        c = wl.config3b()
        return {"A": c["A"], "B": c["B"]}

    c4 = {}
    c5 = {}

    def g4():
        if not c4:
            c4.update(wl.config4())
        return c4

    def g5():
        if not c5:
            c5.update(wl.config5())
        return c5

    def h4():     # the down projection's input: a stand-in with the distribution of GELU outputs
        return wl.normal((8192, 3072), 0.5, "c4.Hstandin")

    def h5():
        return wl.normal((2048, 14336), 0.3, "c5.Hstandin")

    import torch as _t
    G = fact.ACT_GELU_TANH
    S = fact.ACT_SILU_GATE
    allc = [
        Case("c1.square512", 512, 512, 512, 0, maker=c1),
        Case("c2.square8192+bias", 8192, 8192, 8192, 0, bias=True, maker=c2),
        Case("c3a.batched128x512", 512, 512, 512, 0, batch=128, maker=c3a),
        Case("c3b.largeK", 256, 256, 131072, 0, splitk=True, maker=c3b),
        Case("c4.qkv+bias", 8192, 2304, 768, 1, bias=True,
             maker=lambda: {"A": g4()["X"], "B": g4()["Wqkv"], "bias": g4()["bqkv"]}),
        Case("c4.up+bias+gelu", 8192, 3072, 768, 1, act=G, bias=True,
             maker=lambda: {"A": g4()["X"], "B": g4()["W1"], "bias": g4()["b1"]}),
        Case("c4.down+bias+res", 8192, 768, 3072, 1, bias=True, residual=True,
             maker=lambda: {"A": h4(), "B": g4()["W2"], "bias": g4()["b2"], "R": g4()["R"]}),
        Case("c5.qkv", 2048, 6144, 4096, 1, maker=lambda: {"A": g5()["X"], "B": g5()["Wqkv"]}),
        Case("c5.gate_up_silu", 2048, 28672, 4096, 1, act=S,
             maker=lambda: {"A": g5()["X"], "B": _t.cat([g5()["Wg"], g5()["Wu"]])}),
        Case("c5.down+res", 2048, 4096, 14336, 1, residual=True,
             maker=lambda: {"A": h5(), "B": g5()["Wd"], "R": g5()["R"]}),
    ]
    # the paper's own problem shapes (Section 5.1), a second workload: "p*" = the three GEMM
    # problems, "pb.*" = the blocks' projections at the token counts the paper measures
    pg, pl = {}, {}

    def bg():
        if not pg:
            pg.update(wl.paper_block("gpt"))
        return pg

    def bl():
        if not pl:
            pl.update(wl.paper_block("llama"))
        return pl

    paper = [
        Case("p1.square4096", 4096, 4096, 4096, 0, maker=lambda: dict(wl.paper_square())),
        Case("p3.batched128x512x2048x1024", 512, 2048, 1024, 0, batch=128, maker=lambda: dict(wl.paper_batched())),
        Case("p6.largeK524288", 256, 256, 524288, 0, splitk=True, maker=lambda: dict(wl.paper_large_k())),
        Case("pb.gpt.qkv+bias", 65536, 2304, 768, 1, bias=True, maker=lambda: {"A": bg()["X"], "B": bg()["Wqkv"], "bias": bg()["bqkv"]}),
        Case("pb.gpt.up+bias+gelu", 65536, 3072, 768, 1, act=G, bias=True, maker=lambda: {"A": bg()["X"], "B": bg()["W1"], "bias": bg()["b1"]}),
        Case("pb.gpt.down+bias+res", 65536, 768, 3072, 1, bias=True, residual=True,
             maker=lambda: {"A": wl.normal((65536, 3072), 0.5, "pb.gpt.Hstandin"), "B": bg()["W2"], "bias": bg()["b2"], "R": bg()["R"]}),
        Case("pb.llama.qkv", 32768, 6144, 4096, 1, maker=lambda: {"A": bl()["X"], "B": bl()["Wqkv"]}),
        Case("pb.llama.gate_up_silu", 32768, 28672, 4096, 1, act=S, maker=lambda: {"A": bl()["X"], "B": _t.cat([bl()["W1"], bl()["Wu"]])}),
        Case("pb.llama.down+res", 32768, 4096, 14336, 1, residual=True,
             maker=lambda: {"A": wl.normal((32768, 14336), 0.3, "pb.llama.Hstandin"), "B": bl()["W2"], "R": bl()["R"]}),
        # the attention output projections of the two blocks (not among the paper's fused patterns, but
        # whole blocks run them): activations ~ N(0, 0.5) as a stand-in for attention outputs
        Case("pb.gpt.out+bias+res", 65536, 768, 768, 1, bias=True, residual=True,
             maker=lambda: {"A": wl.normal((65536, 768), 0.5, "pb.gpt.Astandin"), "B": wl.normal((768, 768), 0.02, "pb.gpt.Wo"),
                            "bias": wl.normal((768,), 0.02, "pb.gpt.bo"), "R": bg()["R"]}),
        Case("pb.llama.out+res", 32768, 4096, 4096, 1, residual=True,
             maker=lambda: {"A": wl.normal((32768, 4096), 0.5, "pb.llama.Astandin"), "B": wl.normal((4096, 4096), 0.02, "pb.llama.Wo"),
                            "R": bl()["R"]}),
        Case("pc.gpt.out+bias+res", 8192, 768, 768, 1, bias=True, residual=True,
             maker=lambda: {"A": wl.normal((8192, 768), 0.5, "pc.gpt.Astandin"), "B": wl.normal((768, 768), 0.02, "pb.gpt.Wo"),
                            "bias": wl.normal((768,), 0.02, "pb.gpt.bo"), "R": g4()["R"]}),
        Case("pc.llama.out+res", 2048, 4096, 4096, 1, residual=True,
             maker=lambda: {"A": wl.normal((2048, 4096), 0.5, "pc.llama.Astandin"), "B": wl.normal((4096, 4096), 0.02, "pb.llama.Wo"),
                            "R": g5()["R"]}),
    ]
    if names:
        return [c for c in allc + paper if any(c.name.startswith(n) for n in names)]
    return allc


def time_case(case, steps=30, warmup=30, cfg=-1, split=0, group_m=0, min_warm_ms=20.0, min_timed_ms=10.0):
    """Mean ms per launch with device events on the launch stream, or None if the configuration
    is refused (recorded by the sweep as a launch failure).  Short kernels get more warm-up and
    timed launches (at least min_warm_ms / min_timed_ms of work): the GPU needs tens of
    milliseconds under load to settle its clocks."""
    case.alloc()
    rc = case.run(cfg, split, group_m)
    if rc != 0:
        return None
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(4):
        case.run(cfg, split, group_m)
    b.record()
    torch.cuda.synchronize()
    est = max(a.elapsed_time(b) / 4, 1e-3)
    warmup = min(max(warmup, int(min_warm_ms / est) + 1), 2000)
    steps = min(max(steps, int(min_timed_ms / est) + 1), 1000)
    for _ in range(warmup):
        case.run(cfg, split, group_m)
    torch.cuda.synchronize()
    a.record()
    for _ in range(steps):
        case.run(cfg, split, group_m)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / steps


def operand_copies(case, min_bytes_total=768 << 20):
    """The case's operand set and enough further copies of A, B and C (each with its own workspace
    slot) that together they exceed the 256 MB memory-side cache several times."""
    base = case.alloc()
    sets = max(2, int(-(-min_bytes_total // case.min_bytes)))
    copies = [base]
    for _ in range(sets - 1):
        c = dict(base)
        c["A"], c["B"], c["C"], c["ws"] = base["A"].clone(), base["B"].clone(), torch.empty_like(base["C"]), None
        copies.append(c)
    return copies


def time_case_rotating(case, min_bytes_total=768 << 20, steps=30, warmup=30, cfg=-1, split=0, group_m=0, copies=None,
                       min_warm_ms=20.0, min_timed_ms=10.0):
    """As time_case (the table's choice unless cfg / split / group_m say otherwise), but successive launches use different copies of A, B and
    C, enough copies that a launch never finds its operands in the 256 MB memory-side cache from
    the launch before: the figure for a GEMM whose operands come from HBM (the cases bound by
    memory traffic).  Returns (ms per launch, number of copies)."""
    base = case.alloc()
    if copies is None:
        copies = operand_copies(case, min_bytes_total)
    sets = len(copies)

    def launch(i):
        case.t = copies[i % sets]
        return case.run(cfg, split, group_m)

    try:
        if launch(0) != 0:
            return None, sets
        for i in range(sets):             # every copy gets its workspace before the clock starts
            launch(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(4):
            launch(i)
        b.record()
        torch.cuda.synchronize()
        est = max(a.elapsed_time(b) / 4, 1e-3)
        warmup = min(max(warmup, int(min_warm_ms / est) + 1), 2000)
        steps = min(max(steps, int(min_timed_ms / est) + 1), 1000)
        for i in range(warmup):
            launch(i)
        torch.cuda.synchronize()
        a.record()
        for i in range(steps):
            launch(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps, sets
    finally:
        case.t = base


class AttnCase:
    """Causal attention on a packed QKV projection output, through fact_attention."""

    def __init__(self, name, maker):
        self.name, self.maker, self.t = name, maker, None

    def alloc(self):
        if self.t is None:
            w = self.maker()
            self.B, self.T, self.Hq, self.Hkv, self.D = w["batch"], w["tokens"], w["q_heads"], w["kv_heads"], w["head_dim"]
            self.t = {"qkv": w["qkv"].cuda(),
                      "O": torch.empty((self.B, self.T, self.Hq * self.D), dtype=torch.bfloat16, device="cuda")}
        return self.t

    def free(self):
        self.t = None

    @property
    def flops(self):
        """Multiply-adds of the unmasked half only: 2 contractions x 2 x D per (query, visible key) pair."""
        return 4.0 * self.B * self.Hq * self.D * (self.T * (self.T + 1) / 2.0)

    @property
    def min_bytes(self):
        return 2.0 * self.B * self.T * (self.Hq + 2 * self.Hkv) * self.D + 2.0 * self.B * self.T * self.Hq * self.D

    def run(self):
        t = self.alloc()
        W = (self.Hq + 2 * self.Hkv) * self.D
        st = (self.T * W, W, self.D)
        base = t["qkv"].data_ptr()
        return fact.fact_attention(self.B, self.T, self.Hq, self.Hkv, self.D, base, st, base + 2 * self.Hq * self.D, st,
                                   base + 2 * (self.Hq + self.Hkv) * self.D, st, t["O"],
                                   (self.T * self.Hq * self.D, self.Hq * self.D, self.D), 1, 0.0)


def attention_cases():
    import workloads as wl
    return [AttnCase("att4.gpt_8x1024_12h64", lambda: wl.attention4()),
            AttnCase("att5.llama_1x2048_32q8kv128", lambda: wl.attention5(1)),
            AttnCase("att5.llama_16x2048_32q8kv128", lambda: wl.attention5(16))]


def time_attention(steps=30, warmup=30):
    out = {}
    for c in attention_cases():
        c.alloc()
        if c.run() != 0:
            out[c.name] = {"error": "refused"}
            continue
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(4):
            c.run()
        b.record()
        torch.cuda.synchronize()
        est = max(a.elapsed_time(b) / 4, 1e-3)
        w = min(max(warmup, int(20.0 / est) + 1), 2000)
        n = min(max(steps, int(10.0 / est) + 1), 1000)
        for _ in range(w):
            c.run()
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            c.run()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / n
        r = report(c, ms)
        r["flops_counted"] = "causal half: 4 B Hq D T(T+1)/2"
        out[c.name] = r
        c.free()
    return out


def time_blocks(steps=20, warmup=10):
    """Whole decoder blocks through fact_block_forward: ms per block and the TFLOP/s of its matrix
    work (the four projections' 2 M N K plus the attention's causal half)."""
    import workloads as wl
    out = {}
    for name, kind, B, T in (("blk.gpt_8x1024", "gpt", 8, 1024), ("blk.gpt_128x512", "gpt", 128, 512),
                             ("blk.llama_1x2048", "llama", 1, 2048), ("blk.llama_16x2048", "llama", 16, 2048)):
        desc, t, X = wl.block_weights(kind, B, T)
        act = fact.ACT_SILU_GATE if desc["act_gated"] else fact.ACT_GELU_TANH
        b = fact.Block(B, T, desc["d_model"], desc["q_heads"], desc["kv_heads"], desc["head_dim"], desc["d_ff"], int(desc["rms"]),
                       act, int(desc["rope"]), desc["eps"], desc["rope_base"], **{k: v.cuda() for k, v in t.items()})
        need = fact.fact_block_scratch_bytes(b)
        scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
        Xd = X.cuda()
        Y = torch.empty_like(Xd)
        run = lambda: fact.fact_block_forward(b, Xd, Y, scratch, need)
        if run() != 0:
            out[name] = {"error": "refused"}
            continue
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            run()
        e.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(e) / steps
        Tt, d, dff = B * T, desc["d_model"], desc["d_ff"]
        nq, nkv = desc["q_heads"] * desc["head_dim"], desc["kv_heads"] * desc["head_dim"]
        flops = 2.0 * Tt * d * (nq + 2 * nkv) + 2.0 * Tt * nq * d + 2.0 * Tt * d * dff * (3 if desc["act_gated"] else 2) \
            + 4.0 * B * desc["q_heads"] * desc["head_dim"] * (T * (T + 1) / 2.0)
        out[name] = {"ms": round(ms, 4), "tflops": round(flops / ms / 1e9, 1), "pct_mfma_peak": round(100 * flops / ms / 1e9 / PEAK_BF16_TFLOPS, 2),
                     "launches": 10 if desc["rope"] else 9, "scratch_MB": round(need / 2 ** 20, 1)}
        del scratch, Xd, Y, b
    return out


def report(case, ms):
    tf = case.flops / (ms * 1e-3) / 1e12
    gbs = case.min_bytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 5), "tflops": round(tf, 2), "pct_mfma_peak": round(100 * tf / PEAK_BF16_TFLOPS, 2),
            "min_traffic_GBs": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / PEAK_HBM_GBS, 2)}


def time_all(steps=30, warmup=30, names=None):
    out = {}
    for c in cases(names):
        ms = time_case(c, steps, warmup)
        rc, cfg, split = fact.fact_select_config(c.batch, c.M, c.N, c.K, c.trans_b, c.act)
        r = report(c, ms) if ms else {"error": "refused"}
        r["config_id"], r["split_k"] = cfg, split          # split_k < 0: tail split of that many K ranges
        if ms and c.name.startswith("c"):                  # also with operands that miss the memory-side cache (what a GEMM meets inside a block)
            ms_rot, sets = time_case_rotating(c)
            if ms_rot:
                rr = report(c, ms_rot)
                r["rotating_operands"] = {"copies": sets, "ms": rr["ms"], "tflops": rr["tflops"],
                                          "min_traffic_GBs": rr["min_traffic_GBs"], "pct_hbm_peak": rr["pct_hbm_peak"]}
        out[c.name] = r
        c.free()
    return out
