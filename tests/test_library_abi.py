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
    assert len(dh.op_names(dh.DH_ARCH_LLAMA_CP, 0)) == 13 and len(dh.op_names(dh.DH_ARCH_LLAMA_CP, 1)) == 16
    assert dh.op_names(dh.DH_ARCH_LLAMA_CP, 0)[3] == "F_CP_KV" and dh.op_names(dh.DH_ARCH_LLAMA_CP, 1)[10] == "B_CP_DKV"
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
