"""The C-ABI library loads, exports every symbol the header declares, and its
host-only entry points (graph arithmetic, argument validation) behave.  No GPU."""
import os
import re
import ctypes as C
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2510_23264_amd as p
    if not os.path.exists(os.path.join(ROOT, "paper_2510_23264_amd", "libpahq.so")):
        from paper_2510_23264_amd import build
        build.build()
    return p


def test_every_declared_symbol_is_exported():
    p = _lib()
    hdr = open(os.path.join(ROOT, "include", "pahq.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pahq_[a-z_0-9]+)\s*\(", hdr))
    assert {"pahq_init_model", "pahq_clean_cache", "pahq_eval_edges", "pahq_acdc_sweep"} <= names
    lib = p.lib()
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_graph_helpers_match_the_oracle_graph():
    p = _lib()
    from oracle.graph import Graph
    for name in ("cfg1", "cfg2", "cfg3"):
        s = synth.make_shape(name)
        cfg = p.Config.from_shape(s)
        g = Graph(s.n_layers, s.n_heads, s.d_mlp > 0)
        assert p.n_senders(cfg) == g.n_senders and p.n_receivers(cfg) == g.n_receivers
        assert p.edge_count(cfg) == g.n_edges()
        for r in (0, 1, g.n_receivers // 2, g.n_receivers - 2, g.OUT):
            assert p.n_upstream(cfg, r) == g.n_upstream(r)
            assert p.node_of_receiver(cfg, r) == g.node_of_receiver(r)
            assert p.edge_id(cfg, g.n_upstream(r) - 1, r) == g.edge_id(g.n_upstream(r) - 1, r)
    for name, n in (("cfg4", 231877), ("cfg5", 1592881)):
        assert p.edge_count(p.Config.from_shape(synth.make_shape(name))) == n


def test_argument_validation_without_a_device():
    p = _lib()
    s = synth.make_shape("cfg1")
    cfg = p.Config.from_shape(s)
    with pytest.raises(p.PahqError) as e:
        p.n_upstream(cfg, 10 ** 6)
    assert e.value.code == -1
    with pytest.raises(p.PahqError) as e:
        p.edge_id(cfg, 5, 0)                  # sender 5 is not upstream of receiver 0
    assert e.value.code == -1
    bad = p.Config.from_shape(s); bad.n_layers = 0
    with pytest.raises(p.PahqError):
        p.edge_count(bad)
    coarse = p.Config.from_shape(s, split_qkv=False)             # one input per head: a third of the head receivers
    assert p.n_receivers(coarse) == s.n_layers * (s.n_heads + (1 if s.d_mlp else 0)) + 1 and p.workspace_bytes(coarse, 8, 16) > 0
    assert p.edge_count(p.Config.from_shape(synth.make_shape("cfg3"), split_qkv=False)) == 11611
    unsup = p.Config.from_shape(s); unsup.n_heads = 65           # sets of heads are 64-bit masks
    with pytest.raises(p.PahqError) as e:
        p.workspace_bytes(unsup, 8, 16)
    assert e.value.code == -6
    odd = p.Config.from_shape(synth.make_shape("cfg2")); odd.d_mlp = 2050      # hidden rows must be 16-byte multiples
    with pytest.raises(p.PahqError) as e:
        p.workspace_bytes(odd, 8, 16)
    assert e.value.code == -6
    assert p.workspace_bytes(cfg, 8, 16) > 0
    # the all-fp32 mode needs room for unquantised rows of every receiver group
    assert p.workspace_bytes(p.Config.from_shape(s, precision=p.ALL_FP32), 8, 16) > p.workspace_bytes(cfg, 8, 16)
    # fp32 masters on the host: a smaller workspace for deep models, refused with the all-fp32 mode and for other values
    deep = synth.make_shape("cfg3")
    assert p.workspace_bytes(p.Config.from_shape(deep, fp32_on_host=True), 8, 16) < p.workspace_bytes(p.Config.from_shape(deep), 8, 16)
    with pytest.raises(p.PahqError) as e:
        p.workspace_bytes(p.Config.from_shape(s, precision=p.ALL_FP32, fp32_on_host=True), 8, 16)
    assert e.value.code == -6
    wrong = p.Config.from_shape(s); wrong.fp32_residency = 2
    with pytest.raises(p.PahqError) as e:
        p.workspace_bytes(wrong, 8, 16)
    assert e.value.code == -1
    assert p.lib().pahq_prefetch_heads(None, 0, 1) == -1 and p.lib().pahq_get_transfer_stats(None, None) == -1
    assert p.lib().pahq_acdc_sweep_resume(None, C.c_float(0.1), None, 0, None, None, None, 0) == -1
    assert p.lib().pahq_strerror(-3) == b"workspace too small"
    # null handles are rejected, not dereferenced
    assert p.lib().pahq_clean_cache(None, None, None) == -1
    assert p.lib().pahq_eval_edges(None, 0, None, 0, None) == -1
    assert p.lib().pahq_acdc_sweep(None, C.c_float(0.1), None, 0, None, None, None, 0) == -1
