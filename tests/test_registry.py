"""The persisted tuning registry (host logic only, no GPU): file format, the table generated from it,
and the library's run-time loader (the sweep that fills it is exercised on the GPU in
tests/test_gpu_sweep.py)."""
import os

import pytest

import paper_2604_26666_amd as fact
from paper_2604_26666_amd import registry


def test_shipped_registry_parses_and_names_existing_configurations():
    ents = registry.read()
    assert len(ents) >= 10
    n = fact.fact_num_configs()
    for e in ents:
        assert (e.rule, e.dtype, e.arch) == ("gemm", "bf16", "gfx950")
        assert 0 <= e.config < n and (e.split_k == 1 or e.split_k > 1 or e.split_k <= -2) and e.group_m >= 1
        assert e.ms > 0 and e.tflops > 0 and e.build.startswith("v") and e.name != "-"
    # every benchmark configuration has its entry
    names = {e.name for e in ents}
    for want in ("c1.square512", "c2.square8192+bias", "c3a.batched128x512", "c3b.largeK", "c4.qkv+bias", "c4.up+bias+gelu",
                 "c4.down+bias+res", "c5.qkv", "c5.gate_up_silu", "c5.down+res"):
        assert want in names, want
    # an entry that needs a workspace is followed by one of the same shape that does not
    for i, e in enumerate(ents):
        if e.split_k != 1:
            assert i + 1 < len(ents) and ents[i + 1].key == e.key and ents[i + 1].split_k == 1, e.name


def test_compiled_table_is_generated_from_the_registry():
    assert open(registry.TABLE_INC).read() == registry.table_inc(registry.read()), \
        "csrc/tile_table.inc is stale: run python -m paper_2604_26666_amd.registry and rebuild"


def test_library_table_matches_the_registry():
    seen = set()
    for e in registry.read():
        if e.key in seen:
            continue                      # later entries of a shape: the no-workspace alternative
        seen.add(e.key)
        rc, cfg, split = fact.fact_select_config(e.batch, e.M, e.N, e.K, e.trans_b, fact.ACT_SILU_GATE if e.gated else fact.ACT_NONE)
        assert rc == 0 and (cfg, split) == (e.config, e.split_k), f"{e.name}: library says {(cfg, split)}, registry {(e.config, e.split_k)}"


def test_format_round_trip_and_merge():
    ents = registry.read()
    again = registry.parse(registry.render(ents))
    assert [e.line() for e in again] == [e.line() for e in ents]
    new = registry.Entry(1, 8192, 8192, 8192, 0, 0, 3, 1, 2, ms=1.0, tflops=1099.5, build="v999", name="c2.square8192+bias")
    merged = registry.merge(ents, [new])
    assert [e for e in merged if e.key == new.key] == [new] and len(merged) <= len(ents)
    with pytest.raises(ValueError):
        registry.parse("gemm bf16 gfx950 1 64 64 64 kn plain 0 1 1\n")            # no format line
    with pytest.raises(ValueError):
        registry.parse("# fact-registry 2\n")


def test_runtime_loader_overrides_the_compiled_table(tmp_path):
    fact.fact_registry_clear()
    shape = (1, 8192, 8192, 8192, 0, fact.ACT_NONE)
    rc, cfg0, split0 = fact.fact_select_config(*shape)
    assert rc == 0
    other = 3 if cfg0 != 3 else 0
    f = tmp_path / "mine.reg"
    f.write_text("# fact-registry 1\n"
                 "# a comment\n"
                 f"gemm bf16 gfx950 1 8192 8192 8192 kn plain {other} 1 2 0.9 1200.0 vtest mine\n"
                 "gemm bf16 gfx90a 1 8192 8192 8192 kn plain 1 1 2\n"          # another architecture: skipped
                 "gemm fp16 gfx950 1 8192 8192 8192 kn plain 1 1 2\n"          # another data type: skipped
                 "gemm bf16 gfx950 1 64 64 64 kn plain 9999 1 2\n"             # no such configuration: skipped
                 "gemm bf16 gfx950 1 4096 1024 2048 nk gated 0 -2 4\n"
                 "gemm bf16 gfx950 1 4096 1024 2048 nk gated 0 1 4\n"
                 "not an entry at all\n")
    try:
        assert fact.fact_registry_load(str(f)) == 3 and fact.fact_registry_size() == 3
        assert fact.fact_select_config(*shape)[1:] == (other, 1)
        assert fact.fact_select_config(1, 4096, 1024, 2048, 1, fact.ACT_SILU_GATE)[1:] == (0, -2)
        # a second file is consulted before the first
        g = tmp_path / "newer.reg"
        g.write_text(f"# fact-registry 1\ngemm bf16 gfx950 1 8192 8192 8192 kn plain {cfg0} 1 4\n")
        assert fact.fact_registry_load(str(g)) == 1
        assert fact.fact_select_config(*shape)[1:] == (cfg0, 1)
    finally:
        fact.fact_registry_clear()
    assert fact.fact_registry_size() == 0 and fact.fact_select_config(*shape)[1:] == (cfg0, split0)


def test_runtime_loader_refusals(tmp_path):
    assert fact.fact_registry_load(None) == -1
    assert fact.fact_registry_load(str(tmp_path / "missing.reg")) == -7
    bad = tmp_path / "bad.reg"
    bad.write_text("gemm bf16 gfx950 1 64 64 64 kn plain 0 1 1\n")
    assert fact.fact_registry_load(str(bad)) == -7
    v2 = tmp_path / "v2.reg"
    v2.write_text("# fact-registry 2\n")
    assert fact.fact_registry_load(str(v2)) == -7
    assert fact.fact_registry_size() == 0
    # the shipped file loads as it is
    try:
        assert fact.fact_registry_load(registry.DEFAULT) == len(registry.read())
    finally:
        fact.fact_registry_clear()
