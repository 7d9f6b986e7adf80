"""The persisted tuning registry: what the on-device sweep found, kept as a small versioned text file.

The paper keeps its verified kernels in a registry keyed by (rule, data type, architecture)
(Section 3), writes tuning results back into it (Section 4.2 Action 6) and reuses them on later
lookups (Section 4.3).  Here an entry is keyed by (rule, dtype, arch, batch, M, N, K, layout,
epilogue class) and holds the winning launch (tile configuration id, split-K factor, tile-row
group) with its provenance (time, TFLOP/s, library build, workload name).  The file shipped with
the library (registry/gemm_bf16_gfx950.reg) is the source of csrc/tile_table.inc, the table
compiled into the library; `fact_registry_load` reads files of the same format at run time.

Format: see include/fact.h (fact_registry_load).  One entry per line; of several entries for one
key the first is the best launch and a later one with split_k == 1 serves calls without a workspace.
"""
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT = os.path.join(HERE, "registry", "gemm_bf16_gfx950.reg")
TABLE_INC = os.path.join(HERE, "csrc", "tile_table.inc")
VERSION = 1

FILE_HEADER = """# fact-registry 1
# rule dtype arch batch M N K layout epilogue config split_k group_m ms TFLOP/s build name
# layout kn: B as [K][N]; nk: B as [N][K].  N counts the contraction's columns (2 x d_ff when gated).
# split_k 1: K whole; > 1: split-K planes; -g: tail split of g K ranges (both need a workspace; the
# entry after such an entry is the best launch with K whole, for calls that bring none).
"""

TABLE_HEADER = """// Per-shape tile-configuration table: {batch, M, N, K, trans_b, gated, config id, split_k, group_m}.
// GENERATED from registry/gemm_bf16_gfx950.reg by paper_2604_26666_amd/registry.py (write_table_inc):
// edit the registry (or re-run the on-device sweep, python -m paper_2604_26666_amd.sweep), not this file.
// split_k > 1: split-K planes; split_k = -g: tail split of g K ranges (both need a workspace; the
// row after such a row is the best plain launch, for calls without one).  Shapes not listed use
// the analytic model in fact_api.hip.  N is the contraction's column count (2 x d_ff when gated).
"""


@dataclass
class Entry:
    batch: int
    M: int
    N: int
    K: int
    trans_b: int
    gated: int
    config: int
    split_k: int
    group_m: int
    ms: float = 0.0
    tflops: float = 0.0
    build: str = "-"
    name: str = "-"
    rule: str = "gemm"
    dtype: str = "bf16"
    arch: str = "gfx950"

    @property
    def key(self):
        return (self.rule, self.dtype, self.arch, self.batch, self.M, self.N, self.K, self.trans_b, self.gated)

    def line(self):
        return (f"{self.rule} {self.dtype} {self.arch} {self.batch} {self.M} {self.N} {self.K} {'nk' if self.trans_b else 'kn'} "
                f"{'gated' if self.gated else 'plain'} {self.config} {self.split_k} {self.group_m} {self.ms:.5f} {self.tflops:.1f} "
                f"{self.build} {self.name.replace(' ', '_')}")


def parse(text):
    """Entries of a registry text, in file order.  Raises ValueError for another format version
    or an entry before the format line; lines that do not parse are skipped, as the library does."""
    out, header = [], False
    for raw in text.splitlines():
        line = raw.strip()
        if not line:
            continue
        if line.startswith("#"):
            parts = line.split()
            if len(parts) >= 3 and parts[1] == "fact-registry":
                if int(parts[2]) != VERSION:
                    raise ValueError(f"registry format {parts[2]}, this reader knows {VERSION}")
                header = True
            continue
        if not header:
            raise ValueError("entry before the '# fact-registry' line")
        f = line.split()
        if len(f) < 12 or f[7] not in ("kn", "nk") or f[8] not in ("plain", "gated"):
            continue
        try:
            e = Entry(rule=f[0], dtype=f[1], arch=f[2], batch=int(f[3]), M=int(f[4]), N=int(f[5]), K=int(f[6]),
                      trans_b=1 if f[7] == "nk" else 0, gated=1 if f[8] == "gated" else 0,
                      config=int(f[9]), split_k=int(f[10]), group_m=int(f[11]),
                      ms=float(f[12]) if len(f) > 12 else 0.0, tflops=float(f[13]) if len(f) > 13 else 0.0,
                      build=f[14] if len(f) > 14 else "-", name=f[15] if len(f) > 15 else "-")
        except ValueError:
            continue
        out.append(e)
    if not header:
        raise ValueError("not a registry file: no '# fact-registry' line")
    return out


def read(path=DEFAULT):
    with open(path) as f:
        return parse(f.read())


def render(entries):
    return FILE_HEADER + "".join(e.line() + "\n" for e in entries)


def write(entries, path=DEFAULT):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(render(entries))


def merge(old, new):
    """Entries of `old` whose key is not in `new`, then `new` (a re-swept shape replaces all its entries)."""
    keys = {e.key for e in new}
    return [e for e in old if e.key not in keys] + list(new)


def table_inc(entries):
    """Text of csrc/tile_table.inc for these entries (gemm / bf16 / gfx950 ones)."""
    rows = []
    for e in entries:
        if (e.rule, e.dtype, e.arch) != ("gemm", "bf16", "gfx950"):
            continue
        rows.append(f"    {{{e.batch}, {e.M}, {e.N}, {e.K}, {e.trans_b}, {e.gated}, {e.config}, {e.split_k}, {e.group_m}}},   "
                    f"// {e.name}: {e.tflops:.1f} TFLOP/s\n")
    return TABLE_HEADER + "".join(rows)


def write_table_inc(entries=None, path=TABLE_INC):
    text = table_inc(read() if entries is None else entries)
    with open(path, "w") as f:
        f.write(text)
    return path


if __name__ == "__main__":
    print(write_table_inc())
