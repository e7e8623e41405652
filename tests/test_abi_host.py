"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
and its host logic (model description, parameter list, workspace plan, argument errors) is right."""
import os
import re

import pytest

import paper_2111_10672_amd as spb
import workloads as wl


def _declared(repo_root):
    text = open(os.path.join(repo_root, "include", "spb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spb_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(repo_root):
    names = _declared(repo_root)
    assert {"spb_forward", "spb_backward_truncated", "spb_grad_buffers"} <= set(names)
    handle = spb.lib()
    for name in names:
        assert hasattr(handle, name), name
    assert set(names) == set(spb.binding.EXPORTS), "binding and header disagree"


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "ragged_mlp_bf16", "cfg3", "cfg4", "cfg5", "small_resnet_bottleneck_bf16",
                                  "mid_resnet_bottleneck_bf16", "small_encoder_bf16", "resnet101_cifar"])
def test_parameter_list_matches_the_workload(name):
    cfg = wl.get_config(name)
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    try:
        assert spb.spb_num_units(m) == wl.unit_count(cfg)
        specs = wl.tensor_specs(cfg)
        assert spb.spb_param_count(m) == len(specs)
        for i, (pname, shape, unit, _init) in enumerate(specs):
            info = spb.spb_param_info(m, i)
            assert (info["name"], info["shape"], info["unit"], info["dtype"]) == (pname, tuple(shape), unit, cfg["dtype"])
    finally:
        spb.spb_model_destroy(m)


def test_workspace_grows_with_depth_and_depth_is_checked():
    cfg = wl.get_config("cfg2")
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    try:
        sizes = [spb.spb_workspace_size(m, k) for k in range(9)]
        assert all(b >= a for a, b in zip(sizes, sizes[1:])) and sizes[8] > sizes[0]
        # one stashed activation (256 x 1024 bf16) per extra unit in the middle of the range
        assert sizes[5] - sizes[4] == 256 * 1024 * 2
        for bad in (-1, 9):
            with pytest.raises(spb.SpbError) as e:
                spb.spb_workspace_size(m, bad)
            assert e.value.code == -2
    finally:
        spb.spb_model_destroy(m)


def test_bad_descriptions_are_refused():
    cfg = wl.get_config("cfg1")
    for patch, code in [({"batch": 0}, -1), ({"dims": [784]}, -1), ({"dims": [783, 16, 10]}, -1),
                        ({"dims": [784, 0, 10]}, -1)]:
        bad = dict(cfg, **patch)
        with pytest.raises(spb.SpbError) as e:
            spb.spb_model_create(spb.desc_from_config(bad))
        assert e.value.code == code and spb.spb_last_error()
    d = spb.desc_from_config(cfg)
    d.family = 17
    with pytest.raises(spb.SpbError):
        spb.spb_model_create(d)


def test_state_errors_without_a_gpu():
    cfg = wl.get_config("tiny_mlp_f32")
    m = spb.spb_model_create(spb.desc_from_config(wl.get_config("ragged_mlp_f32")))
    try:
        with pytest.raises(spb.SpbError) as e:          # backward before any forward
            spb.spb_backward_truncated(m, 1, 0)
        assert e.value.code == -3
        with pytest.raises(spb.SpbError) as e:          # forward with nothing bound: refused before any launch
            spb.spb_forward(m, 256, 256, None, 1, 256, 1 << 30, 256, 0)
        assert e.value.code == -3
        with pytest.raises(spb.SpbError) as e:          # null input
            spb.spb_forward(m, None, 256, None, 1, 256, 1 << 30, 256, 0)
        assert e.value.code == -1
        with pytest.raises(spb.SpbError) as e:
            spb.spb_grad_buffers(m, 1)
        assert e.value.code == -3
        assert spb.spb_grad_buffers(m, 0) == []
        with pytest.raises(spb.SpbError) as e:          # wrong pointer count
            spb.spb_bind_params(m, [256, 512])
        assert e.value.code == -1
        with pytest.raises(spb.SpbError) as e:          # misaligned pointer
            spb.spb_bind_params(m, [256 + 4] * spb.spb_param_count(m))
        assert e.value.code == -1
    finally:
        spb.spb_model_destroy(m)
    del cfg


def test_worker_depth_rule_and_aggregation_argument_errors():
    cfg = wl.get_config("cfg2")
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    try:
        L = wl.unit_count(cfg)
        assert [spb.spb_worker_depth(m, j, 4) for j in range(1, 5)] == [2, 4, 6, 8]
        assert [spb.spb_worker_depth(m, j, 3) for j in range(1, 4)] == [3, 6, 8]      # ceil(8 j / 3)
        assert spb.spb_worker_depth(m, 5, 5) == L
        for j, n in ((0, 4), (5, 4), (1, 0)):
            with pytest.raises(spb.SpbError) as e:
                spb.spb_worker_depth(m, j, n)
            assert e.value.code == -1
        n_params = spb.spb_param_count(m)
        none = [None] * n_params
        with pytest.raises(spb.SpbError) as e:      # too many workers
            spb.spb_aggregate_update(m, [1] * 9, [none] * 9, none, 0.1, 0.9, 0.0, True, 0)
        assert e.value.code == -1
        with pytest.raises(spb.SpbError) as e:      # depth out of range
            spb.spb_aggregate_update(m, [L + 1], [none], none, 0.1, 0.9, 0.0, True, 0)
        assert e.value.code == -2
        with pytest.raises(spb.SpbError) as e:      # parameters not bound
            spb.spb_aggregate_update(m, [1], [none], none, 0.1, 0.9, 0.0, True, 0)
        assert e.value.code == -3
    finally:
        spb.spb_model_destroy(m)


def test_static_workspace_entry_point_checks_its_arguments_on_the_host():
    """Everything spb_forward_static refuses, it refuses before any GPU call."""
    m = spb.spb_model_create(spb.desc_from_config(wl.get_config("cfg2")))
    big = spb.spb_model_create(spb.desc_from_config(wl.get_config("wide_mlp_bf16")))
    try:
        with pytest.raises(spb.SpbError) as e:          # null input
            spb.spb_forward_static(m, None, 256, None, 1, 256, 0)
        assert e.value.code == -1
        with pytest.raises(spb.SpbError) as e:          # depth out of range
            spb.spb_forward_static(m, 256, 256, None, 9, 256, 0)
        assert e.value.code == -2
        with pytest.raises(spb.SpbError) as e:          # nothing bound
            spb.spb_forward_static(m, 256, 256, None, 1, 256, 0)
        assert e.value.code == -3
        assert all(spb.spb_workspace_size(m, k) <= spb.SPB_STATIC_WORKSPACE_BYTES for k in range(9))
        spb.spb_bind_params(big, [256] * spb.spb_param_count(big))
        with pytest.raises(spb.SpbError) as e:          # does not fit the fixed array
            spb.spb_forward_static(big, 256, 256, None, 2, 256, 0)
        assert e.value.code == -4
    finally:
        spb.spb_model_destroy(m)
        spb.spb_model_destroy(big)


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg5", "small_resnet_bottleneck_bf16"])
def test_unit_views_lie_inside_the_workspace_and_have_the_units_shapes(name):
    cfg = wl.get_config(name)
    m = spb.spb_model_create(spb.desc_from_config(cfg))
    try:
        L = spb.spb_num_units(m)
        total = spb.spb_workspace_size(m, L)
        size = {"f32": 4, "bf16": 2, "i32": 4}
        seen = set()
        for u in range(L):
            vin, vg = spb.spb_unit_io(m, L, u)
            assert (vin["offset"] == spb.SPB_VIEW_CALLER_INPUT) == (u == 0)
            assert (vg["offset"] == spb.SPB_VIEW_NONE) == (u == L - 1)
            for v in (vin, vg):
                if v["offset"] >= 0:
                    assert v["offset"] % 256 == 0 and v["pitch"] >= v["cols"] > 0 and v["rows"] > 0
                    assert v["offset"] + ((v["rows"] - 1) * v["pitch"] + v["cols"]) * size[v["dtype"]] <= total
            if vin["offset"] >= 0:
                assert vin["offset"] not in seen            # every unit's input has a buffer of its own at full depth
                seen.add(vin["offset"])
            if u + 1 < L:                                   # what unit u hands up is what unit u + 1 takes in
                up, _ = spb.spb_unit_io(m, L, u + 1)
                assert (vg["rows"], vg["cols"]) == (up["rows"], up["cols"])
        with pytest.raises(spb.SpbError) as e:              # a unit below the cut keeps nothing
            spb.spb_unit_io(m, 2, L - 3)
        assert e.value.code == -1
    finally:
        spb.spb_model_destroy(m)
