"""The C ABI without a GPU: the library loads, exports every symbol the header
declares, and rejects malformed tables / arguments on the host."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2509_25041_amd as grace
from paper_2509_25041_amd import binding
from workloads import CONFIGS, make_workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "grace_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grace_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = grace.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert os.path.dirname(grace.library_path()).endswith("paper_2509_25041_amd")


def test_binding_has_the_entry_points_under_their_own_names():
    """Every exported call is reachable from Python under the C name (functions of the binding, re-exported
    by the package), the table's calls as methods of GraceTable."""
    methods = {"grace_table_create": "__init__", "grace_table_destroy": "destroy", "grace_table_info": "__init__",
               "grace_table_instances": "instances", "grace_table_local_experts": "local_experts",
               "grace_table_set_fold_limits": "set_fold_limits"}
    for n in binding.EXPORTS:
        if n in methods:
            assert callable(getattr(grace.GraceTable, methods[n]))
        else:
            assert callable(getattr(binding, n)), n
            assert getattr(grace, n) is getattr(binding, n), n


def test_valid_tables_pass_validation():
    for cfg in CONFIGS.values():
        pl = make_workload(cfg, T=256).placement
        grace.grace_table_validate(pl.E, pl.R, pl.N, pl.rank_node, pl.poll_weight, pl.inst_ptr, pl.inst_rank)


GOOD = dict(E=2, R=2, N=1, rank_node=[0, 0], poll_weight=[1, 2], inst_ptr=[0, 1, 3], inst_rank=[0, 0, 1])


@pytest.mark.parametrize("patch,status", [
    (dict(poll_weight=[1, 0]), -3),                 # zero weight
    (dict(poll_weight=[1, 70000]), -3),             # oversized weight
    (dict(inst_ptr=[0, 0, 2], inst_rank=[0, 1, 1]), -3),   # expert without instance
    (dict(inst_rank=[0, 0, 2]), -3),                # rank out of range
    (dict(inst_rank=[0, 1, 1]), -3),                # duplicate (expert, rank)
    (dict(inst_rank=[0, 1, 0]), -3),                # unsorted ranks
    (dict(rank_node=[1, 0], N=2), -3),              # decreasing rank_node
    (dict(rank_node=[0, 1]), -3),                   # node id out of range
    (dict(inst_ptr=[1, 2, 3]), -3),                 # inst_ptr not starting at 0
    (dict(E=0), -1),
    (dict(E=300, inst_ptr=list(range(301)), inst_rank=[0] * 300), -2),
])
def test_malformed_tables_are_rejected(patch, status):
    a = {**GOOD, **patch}
    with pytest.raises(grace.GraceError) as ei:
        grace.grace_table_validate(a["E"], a["R"], a["N"], a["rank_node"], a["poll_weight"], a["inst_ptr"],
                                   a["inst_rank"])
    assert ei.value.status == status
    assert grace.grace_last_error() != ""


def test_null_and_range_checks_without_device():
    lib = grace.load_library()
    assert lib.grace_table_validate(2, 2, 1, None, None, None, None) == -1
    assert lib.grace_table_destroy(None) == 0
    assert lib.grace_table_info(None, None, None, None, None, None) == -1
    # compute entry points refuse a null table before touching the device
    assert lib.grace_route(None, 0, 0, None, 1, 1, 1, 1, None, None, None, None, None, None, None, None) == -1
    assert lib.grace_permute(None, None, 1, 1, None, 8, 1, None, None, None, None, None, None, None, None) == -1
    assert lib.grace_expert_ffn(None, 0, None, None, 1, 1, 8, 8, 1, None, None, None, None, None, None) == -1
    assert lib.grace_shared_ffn(None, 1, 8, 8, 0, 1, None, None, None, None, None, None) == -1
    assert lib.grace_shared_ffn(None, 1, 12, 8, 1, 1, None, None, None, None, None, None) == -2   # bf16 needs d % 8 == 0
    assert lib.grace_combine(None, None, None, 1, 1, 3, 1, None, None, None) == -2               # 6-byte rows
    assert lib.grace_combine(None, None, None, 1, 1, 8, 1, None, None, None) == -1               # null pointers
    assert lib.grace_combine(None, None, None, 0, 1, 8, 1, None, None, None) == 0                # nothing to do
    assert lib.grace_mfma_sustained(1, 1, None, None) == -1
    assert lib.grace_table_set_fold_limits(None, -1, -1) == -1
    assert lib.grace_permute_rows(None, None, 1, 1, 8, 1, None, None) == -1
    assert lib.grace_shared_ffn_up_scatter(None, 1, 8, 8, 1, 1, None, None, None, None, 0, None, None) == -1
    assert lib.grace_permute_rows(None, None, 0, 1, 8, 1, None, None) == 0
    assert lib.grace_route_permute_static(None, 0, 0, None, 1, 1, 1, 1, None, None, None, None, None, None, None, 8, 1, None,
                                          None, None, None, None, None, None) == -1
    assert lib.grace_expert_ffn_up_share(None, 0, None, None, 1, 1, 8, 8, 1, None, None, None, None, None) == -1
    assert lib.grace_expert_ffn_down_share(None, 0, None, 1, 1, 8, 8, 1, None, None, None, None, None) == -1
    assert lib.grace_send_lists(None, 0, None, 1, 1, None, None, None, None, None, None, None, None) == -1


def test_workspace_bytes():
    assert grace.grace_workspace_bytes(-1, 8, 2, 11) == 0
    small = grace.grace_workspace_bytes(256, 8, 2, 11)
    assert small >= 2 * 4 * 8 * 4
    big = grace.grace_workspace_bytes(4096, 64, 8, 76, 2048, 1024, 0, grace.GRACE_BF16)
    assert big >= 4096 * 8 * 1024 * 2
    assert grace.grace_workspace_bytes(4096, 64, 8, 76, 2048, 1024, 0, grace.GRACE_F32) >= 2 * (big - 256)
