"""The C-ABI library loads and exports every entry point include/dhelix.h declares; host-only
entry points (planner, argument checks) behave as documented.  No GPU needed."""
import os
import re

import pytest

from paper_2411_15871_amd import dhelix as dh

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "dhelix.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dh_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported_and_bound():
    syms = declared_symbols()
    assert len(syms) >= 30
    for s in syms:
        assert hasattr(dh.lib, s), s
        assert s in dh.SIGNATURES, "binding lacks " + s
        assert hasattr(dh, s), "python wrapper lacks " + s
    assert sorted(dh.SIGNATURES) == syms


def test_op_names_and_error_strings():
    assert dh.FWD_OPS[:4] == ["F_NORM1", "F_QKV", "F_ROPE", "F_ATTN"] and len(dh.FWD_OPS) == 12 and len(dh.BWD_OPS) == 15
    assert len(dh.op_names(dh.DH_ARCH_GPT, 0)) == 13 and len(dh.op_names(dh.DH_ARCH_GPT, 1)) == 16
    assert len(dh.op_names(dh.DH_ARCH_MOE, 0)) == 14 and len(dh.op_names(dh.DH_ARCH_MOE, 1)) == 18
    assert len(dh.op_names(dh.DH_ARCH_LLAMA_CP, 0)) == 13 and len(dh.op_names(dh.DH_ARCH_LLAMA_CP, 1)) == 17
    assert dh.op_names(dh.DH_ARCH_LLAMA_CP, 0)[3] == "F_CP_KV" and dh.op_names(dh.DH_ARCH_LLAMA_CP, 1)[10:12] == ["B_CP_DKV", "B_CP_SEND"]
    assert dh.dh_op_name(0, 0, 99) is None and dh.dh_op_name(0, 2, 0) is None and dh.dh_op_name(7, 0, 0) is None
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_layer_create(arch=0, dtype=1, batch=1, seq=8, hidden=100, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=64,
                           eps=1e-5, rope_base=1e4, n_ranks=1)
    assert e.value.code == dh.DH_ERR_SHAPE and "multiples of 8" in str(e.value)
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_layer_create(arch=0, dtype=1, batch=1, seq=8, hidden=64, n_q_heads=3, n_kv_heads=2, head_dim=64, ffn=64,
                           eps=1e-5, rope_base=1e4, n_ranks=1)
    assert e.value.code == dh.DH_ERR_SHAPE
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_layer_create(arch=7, dtype=1, batch=1, seq=8, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=64,
                           eps=1e-5, rope_base=1e4, n_ranks=1)
    assert e.value.code == dh.DH_ERR_UNSUPPORTED


def test_context_parallel_layer_configuration_is_checked():
    """Host-only checks of the context-parallel layer description: rank range, the bf16 kernels' 128-position grid, and
    the sizes that grow with the rank's position (it attends to cp_rank+1 chunks of keys)."""
    base = dict(arch=dh.DH_ARCH_LLAMA_CP, dtype=dh.DH_BF16, batch=1, seq=256, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=64,
                ffn=64, eps=1e-5, rope_base=1e4, n_ranks=1, cp_ranks=4)
    for bad in (dict(cp_rank=4), dict(cp_rank=-1), dict(cp_ranks=0, cp_rank=0), dict(cp_ranks=17, cp_rank=0),
                dict(cp_rank=1, cross_blocks=-1)):
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_layer_create(**{**base, **bad})
        assert e.value.code == dh.DH_ERR_INVALID_ARG
    with pytest.raises(dh.DhelixError) as e:  # 3 * 200 is not a multiple of 128
        dh.dh_layer_create(**{**base, "seq": 200, "cp_rank": 3})
    assert e.value.code == dh.DH_ERR_SHAPE
    dh.dh_layer_destroy(dh.dh_layer_create(**{**base, "seq": 200, "cp_rank": 3, "dtype": dh.DH_F32}))  # fp32 has no such grid
    sizes = []
    for r in range(4):
        layer = dh.dh_layer_create(**{**base, "cp_rank": r})
        sizes.append((dh.dh_layer_saved_bytes(layer), dh.dh_layer_workspace_bytes(layer, dh.DH_WS_BWD)))
        gf, gb = dh.dh_layer_op_graph(layer, 0), dh.dh_layer_op_graph(layer, 1)
        assert gf.n_ops == 13 and gb.n_ops == 17
        assert [gf.is_comm[i] for i in range(13)].count(2) == 1 and [gb.is_comm[i] for i in range(17)].count(2) == 2
        assert sum(gb.side_ok[i] for i in range(17)) == 4
        deps_f = [(gf.dep_src[e], gf.dep_dst[e]) for e in range(gf.n_deps)]
        assert not any(d == dh.op_names(dh.DH_ARCH_LLAMA_CP, 0).index("F_CP_KV") for _, d in deps_f)  # the exchange waits for nothing
        dh.dh_layer_destroy(layer)
    assert all(a[0] < b[0] and a[1] < b[1] for a, b in zip(sizes, sizes[1:]))  # one more chunk of keys and key gradients per rank
    plain = dh.dh_layer_create(**{**base, "arch": dh.DH_ARCH_LLAMA, "cp_ranks": 0})
    assert dh.dh_layer_saved_bytes(plain) < sizes[0][0]
    dh.dh_layer_destroy(plain)
