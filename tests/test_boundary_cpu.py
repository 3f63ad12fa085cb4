"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, partitions bit-exactly like the oracle, and rejects bad arguments."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as O
import paper_2009_09523_amd as vf
from paper_2009_09523_amd import binding
import vf_inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_in_header():
    text = open(os.path.join(ROOT, "include", "vf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    declared = _declared_in_header()
    assert declared == vf.exported_symbols()
    L = C.CDLL(vf.lib_path())
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("sizes", [[16] * 4, [48, 48, 32, 32, 16, 16, 48, 16], [1], [7, 1, 300], [128] * 64,
                                   [3, 5, 7, 11, 13]])
def test_partition_bit_exact_with_oracle(sizes):
    B = sum(sizes)
    off, w = vf.vf_partition(sizes, B)
    o_off, o_w = O.partition(sizes, B)
    assert off.dtype == o_off.dtype == np.int32
    assert off.tobytes() == o_off.tobytes()
    assert w.tobytes() == o_w.tobytes()


@pytest.mark.parametrize("sizes,B", [([], 0), ([0, 4], 4), ([3, 3], 7), ([-1, 5], 4), ([4], 0)])
def test_partition_rejects(sizes, B):
    with pytest.raises(vf.VfError) as e:
        vf.vf_partition(sizes, B)
    assert e.value.code == binding.VF_EINVAL


def test_partition_null_and_untouched_outputs():
    L = vf.lib()
    assert L.vf_partition(None, 2, 4, None, None) == binding.VF_EINVAL
    sizes = (C.c_int32 * 2)(3, 2)
    off = (C.c_int32 * 3)(-7, -7, -7)
    assert L.vf_partition(sizes, 2, 6, off, None) == binding.VF_EINVAL
    assert list(off) == [-7, -7, -7]
    assert L.vf_partition(sizes, 2, 5, off, None) == binding.VF_OK
    assert list(off) == [0, 3, 5]


def _cfg(**kw):
    cfg = binding.config_from_workload(I.workload("C1"))
    for k, v in kw.items():
        setattr(cfg, k, v)
    return cfg


@pytest.mark.parametrize("kw", [dict(dtype=7), dict(optimizer=3), dict(max_nodes=0), dict(max_node_size=0),
                                dict(n_dims=1), dict(n_dims=17), dict(model_kind=5),
                                dict(max_node_size=100, max_batch=64), dict(node_group=3), dict(node_group=64),
                                dict(node_group=-1), dict(fold_window=9)])
def test_init_rejects_bad_config_before_touching_the_device(kw):
    h = C.c_void_p(123)
    cfg = _cfg(**kw)
    assert vf.lib().vf_init(C.byref(cfg), C.byref(h)) == binding.VF_EINVAL
    assert not h.value


def test_init_null_arguments():
    L = vf.lib()
    h = C.c_void_p()
    assert L.vf_init(None, C.byref(h)) == binding.VF_EINVAL
    assert L.vf_step(None, None, None, None, 1, 1, None) == binding.VF_EINVAL
    assert L.vf_grads(None, None) == binding.VF_EINVAL
    assert L.vf_num_params(None) == 0
    L.vf_destroy(None)
    assert L.vf_strerror(binding.VF_EINVAL).decode() == "invalid argument"


def test_bf16_mlp_needs_16_byte_rows():
    wl = I.Workload(name="odd", kind="mlp", dims=(100, 16, 4), batchnorm=False, node_sizes=(4,),
                    dtype="bf16")
    cfg = binding.config_from_workload(wl)
    h = C.c_void_p()
    assert vf.lib().vf_init(C.byref(cfg), C.byref(h)) == binding.VF_EINVAL


def test_state_size_of_a_null_context_is_zero_and_config_rejects_a_bad_share():
    import ctypes as C
    assert vf.lib().vf_state_bytes(None) == 0
    from paper_2009_09523_amd.binding import config_from_workload
    import vf_inputs as I
    from dataclasses import replace
    cfg = config_from_workload(replace(I.workload("mlp_small_bn_f32"), bn_momentum=1.5))
    h = C.c_void_p()
    assert vf.lib().vf_init(C.byref(cfg), C.byref(h)) != 0 and not h


def test_prefetch_entry_points_reject_null_arguments_without_a_device():
    assert vf.lib().vf_prefetch(None, None, None, 4) != 0
    assert vf.lib().vf_step_prefetched(None, None, 1, None) != 0


@pytest.mark.parametrize("kw", [dict(width=12), dict(width=512), dict(width=0), dict(img=0), dict(in_ch=0),
                                dict(classes=0), dict(n_blocks=-1), dict(dtype=binding.VF_F32)])
def test_conv_config_rejects_what_the_kernels_do_not_take(kw):
    """Width a multiple of 8 up to 256 (16-byte channel vectors, one column group per four
    channels), bf16 only."""
    cfg = binding.config_from_workload(I.workload("conv_tiny_bf16"))
    for k, v in kw.items():
        setattr(cfg, k, v)
    h = C.c_void_p(123)
    assert vf.lib().vf_init(C.byref(cfg), C.byref(h)) == binding.VF_EINVAL
    assert not h.value


def test_null_context_queries():
    L = vf.lib()
    assert L.vf_streams(None) == 0 and L.vf_fold_window(None) == 0
    cfg = _cfg(fold_window=9)
    h = C.c_void_p(5)
    assert L.vf_init(C.byref(cfg), C.byref(h)) == binding.VF_EINVAL and not h.value


def test_config_struct_matches_the_header_field_for_field():
    """The binding's structure lists the fields of vf_config in the header's order."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "vf.h")).read()
    body = text[text.index("typedef struct vf_config {"):text.index("} vf_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip().replace("typedef struct vf_config {", "").strip()
        parts = decl.split(None, 1)
        if len(parts) < 2:
            continue
        for n in parts[1].split(","):
            names.append(re.sub(r"\[.*\]", "", n.strip().lstrip("*")))
    assert names == [f[0] for f in binding.VfConfig._fields_]
