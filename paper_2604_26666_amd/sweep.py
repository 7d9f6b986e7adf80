"""On-device sweep: time every compiled tile configuration on the benchmark shapes, keep the
winners in the persisted registry and regenerate the table compiled into the library.

This is the auto-tuning step of the paper (Section 4.2 Action 5; methodology in Section 5.1: each
configuration is run with warm-up and timed iterations, configurations that cannot run are
recorded as launch failures) followed by the registry write of Action 6, reduced to what this
library needs: (rule, dtype, arch, shape, layout, epilogue class) -> (tile configuration, split-K
factor, tile-row group) with time, TFLOP/s and the library build that measured it.

Parity gate.  A candidate is accepted only if its output agrees with a reference the product
forms itself, without any tile configuration: the guarded one-thread-per-element kernel
(FACT_CONFIG_GUARDED), run once per shape.  That kernel adds the same products in fp32 in plain
ascending order, so agreement is demanded at the scale of the matrix (2^-6 of the largest
magnitude per element, 4e-3 in relative Frobenius norm).  Among the candidates that keep K whole
the first accepted one then serves as a bit-level reference: every configuration adds the
same products in the same order, so their outputs must be identical bit for bit.  (The tests hold
the table's choices, and the winner of a swept case, to the CPU oracle; the sweep itself does not
know the oracle.)

Run on a machine with the GPU:  python -m paper_2604_26666_amd.sweep [case-prefix ...]
Then rebuild the library (python -m paper_2604_26666_amd.build): it compiles csrc/tile_table.inc,
which this tool regenerates from the registry file.  The raw per-candidate log goes to the file
the environment variable FACT_SWEEP_LOG names (default: fact_sweep_log.json in the system's
temporary directory; it is not kept in the repository).
"""
import json
import os
import sys

import torch

from . import binding as fact
from . import registry
from . import workbench as wb

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
RAW_LOG = os.environ.get("FACT_SWEEP_LOG") or os.path.join(__import__("tempfile").gettempdir(), "fact_sweep_log.json")
CONFIG_GUARDED = -2


def _bits(t):
    return t.view(torch.int16)


def _close(out, ref):
    """Agreement at the scale of the matrix (different summation order or split)."""
    a, b = out.float(), ref.float()
    scale = float(b.abs().max()) + 1e-30
    return bool(torch.isfinite(a).all() and (a - b).abs().max() <= 2.0 ** -6 * scale and (a - b).norm() <= 4e-3 * b.norm() + 1e-30)


REF_FLOPS_LIMIT = 2.0e12      # above this the guarded kernel covers a sample of rows (it runs at a few TFLOP/s)
REF_BLOCK = 256


def guarded_reference(case):
    """(rows, result on those rows) from the guarded kernel, or None if it refuses (then nothing is
    accepted).  Small problems: every row of every batch entry.  Large ones: blocks of 256 rows
    spread over M (first, last and evenly between), each computed by a guarded launch on the
    operand rows themselves."""
    t = case.alloc()
    nout, M = case.nout, case.M
    if case.flops <= REF_FLOPS_LIMIT or case.batch > 1 or M <= 4 * REF_BLOCK:
        t["C"].fill_(0)
        rc = case.run(cfg=CONFIG_GUARDED, split=1)
        torch.cuda.synchronize()
        return (None, t["C"].clone()) if rc == 0 else None
    nblk = max(2, min(8, int(REF_FLOPS_LIMIT / (2.0 * REF_BLOCK * case.N * case.K))))
    starts = sorted({int(round(i * (M - REF_BLOCK) / (nblk - 1))) for i in range(nblk)})
    rows = torch.cat([torch.arange(s0, s0 + REF_BLOCK) for s0 in starts]).cuda()
    out = torch.zeros((len(starts) * REF_BLOCK, nout), dtype=torch.bfloat16, device="cuda")
    ldb = case.K if case.trans_b else case.N
    for i, s0 in enumerate(starts):
        R = t.get("R")
        ep = fact.Epilogue(bias=t.get("bias"), residual=None if R is None else R[s0:], ldr=nout, act=case.act)
        rc = fact.fact_gemm_ex(1, REF_BLOCK, case.N, case.K, t["A"][s0:], case.K, 0, t["B"], ldb, 0, case.trans_b,
                               out[i * REF_BLOCK:], nout, 0, ep, CONFIG_GUARDED, 1, 0, None, 0)
        if rc != 0:
            return None
    torch.cuda.synchronize()
    return rows, out


def _on_rows(out, rows):
    return out if rows is None else out.index_select(0, rows)


def sweep_case(case, steps=20, warmup=20, groups=(1, 2, 4, 8, 16), splits=(2, 4, 8, 16, 32, 64, 128), tails=(-2, -3, -4),
               configs=None):
    """Returns (accepted candidates sorted by time, failures).  configs: ids to try (default: all)."""
    case.alloc()
    got = guarded_reference(case)
    if got is None:
        return [], [{"cfg": CONFIG_GUARDED, "split": 1, "group_m": 0, "reason": "the guarded kernel refused the shape: no reference"}]
    rows, ref = got
    ids = range(fact.fact_num_configs()) if configs is None else configs
    results, failures = [], []
    # Large-K cases are bound by memory traffic: every operand byte is read once, so what matters is
    # the time with operands that come from HBM.  They are timed with the operands rotated through
    # copies larger than the memory-side cache (each copy's output is checked like any other).
    copies = wb.operand_copies(case) if case.splitk else None
    whole_ref = None                         # first accepted output with K whole: the bit-level reference
    split_list = [1] + [t for t in tails if case.batch == 1] + [s for s in splits if case.splitk and case.K // s >= 256]
    for cfg in ids:
        for split in split_list:
            for g in groups:
                case.t["C"].fill_(0)
                if copies is None:
                    ms = wb.time_case(case, steps, warmup, cfg, split, g, min_warm_ms=6.0, min_timed_ms=8.0)
                else:
                    ms, _ = wb.time_case_rotating(case, steps=steps, warmup=warmup, cfg=cfg, split=split, group_m=g, copies=copies,
                                                  min_warm_ms=6.0, min_timed_ms=8.0)
                if ms is None:
                    failures.append({"cfg": cfg, "split": split, "group_m": g, "reason": "refused"})
                    break
                out = case.t["C"]
                if not _close(_on_rows(out, rows), ref):
                    failures.append({"cfg": cfg, "split": split, "group_m": g, "reason": "differs from the guarded kernel's result"})
                    continue
                if split == 1:
                    if whole_ref is None:
                        whole_ref = out.clone()
                    elif not torch.equal(_bits(out), _bits(whole_ref)):
                        failures.append({"cfg": cfg, "split": split, "group_m": g, "reason": "bits differ from another configuration with K whole"})
                        continue
                results.append({"cfg": cfg, "split": split, "group_m": g, "ms": ms})
    results.sort(key=lambda r: r["ms"])
    return results, failures


def entries_for(case, results):
    """Registry entries of a swept case: the best launch and, if that one needs a workspace, the best with K whole."""
    if not results:
        return []
    build = f"v{fact.fact_version()}"
    gated = 1 if case.act == fact.ACT_SILU_GATE else 0

    def entry(r):
        rep = wb.report(case, r["ms"])
        return registry.Entry(case.batch, case.M, case.N, case.K, int(case.trans_b), gated, r["cfg"], r["split"], r["group_m"],
                              ms=r["ms"], tflops=rep["tflops"], build=build, name=case.name)

    out = [entry(results[0])]
    if results[0]["split"] != 1:
        plain = next((r for r in results if r["split"] == 1), None)
        if plain:
            out.append(entry(plain))
    return out


def main(argv):
    names = argv or None
    new, log = [], {}
    for case in wb.cases(names):
        res, fail = sweep_case(case)
        case.free()
        if not res:
            print(f"{case.name}: no configuration was accepted ({len(fail)} failures)", flush=True)
            log[case.name] = {"failed": fail}
            continue
        ents = entries_for(case, res)
        new += ents
        best = res[0]
        print(f"{case.name}: best cfg {best['cfg']} {fact.fact_config_info(best['cfg'])} split {best['split']} "
              f"group_m {best['group_m']}: {ents[0].tflops} TFLOP/s; {len(res)} accepted, {len(fail)} failed", flush=True)
        log[case.name] = {"best": best, "top": res[:8], "accepted": len(res), "failed": fail}
    old = registry.read() if os.path.exists(registry.DEFAULT) else []
    merged = registry.merge(old, new)
    registry.write(merged)
    registry.write_table_inc(merged)
    os.makedirs(os.path.dirname(os.path.abspath(RAW_LOG)), exist_ok=True)
    prev = {}
    if os.path.exists(RAW_LOG):
        try:
            prev = json.load(open(RAW_LOG))
        except Exception:
            prev = {}
    prev.update(log)
    json.dump(prev, open(RAW_LOG, "w"), indent=1)
    print("wrote", registry.DEFAULT, "and", registry.TABLE_INC)


if __name__ == "__main__":
    main(sys.argv[1:])
