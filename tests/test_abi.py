"""The C boundary without a GPU: the built library loads, exports every function the header
declares, the Python binding's structures mirror the header's field by field, and the host-side
argument checks (which run before anything touches a device) answer with the documented codes.
No compute call is made here."""
import ctypes as C
import os
import re

import pytest

import paper_2503_14153_amd as sd
from paper_2503_14153_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "specdec.h")).read()


def _strip_comments(text: str) -> str:
    return re.sub(r"/\*.*?\*/", "", text, flags=re.S)


def _declared_functions():
    code = _strip_comments(HEADER)
    return re.findall(r"^(?:int|size_t|const char\s*\*)\s+(sd_\w+)\s*\(", code, flags=re.M)


def _struct_fields(name: str):
    code = _strip_comments(HEADER)
    body = re.search(r"typedef struct %s\s*\{(.*?)\}\s*%s\s*;" % (name, name), code, flags=re.S).group(1)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        names = decl.split(",")
        fields.append(re.search(r"(\w+)\s*$", names[0]).group(1))
        fields += [re.search(r"(\w+)\s*$", n).group(1) for n in names[1:]]
    return fields


def _defines():
    """Integer constants of the header: #define'd ones and the enumerators of sd_status."""
    code = _strip_comments(HEADER)
    d = {k: int(v) for k, v in re.findall(r"^#define\s+(SD_\w+)\s+\(?(-?\d+)\)?\s*$", code, flags=re.M)}
    d.update({k: int(v) for k, v in re.findall(r"^\s*(SD_\w+)\s*=\s*(-?\d+)\s*,?\s*$", code, flags=re.M)})
    return d


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2503_14153_amd import build
        build.build(verbose=False)
    return sd.lib()


def test_header_declares_what_the_binding_lists():
    declared = _declared_functions()
    assert len(declared) == len(set(declared)) and len(declared) >= 27
    assert sorted(declared) == sorted(sd.EXPORTED_SYMBOLS)


def test_library_exports_every_declared_function(lib):
    for name in _declared_functions():
        assert getattr(lib, name) is not None, name


@pytest.mark.parametrize("cname,ctype", [("sd_config", binding._Config), ("sd_weights", binding._Weights),
                                         ("sd_step_io", binding._StepIO), ("sd_typical", binding._Typical)])
def test_binding_structures_mirror_the_header(cname, ctype):
    assert _struct_fields(cname) == [f[0] for f in ctype._fields_]


def test_error_codes_match_the_binding():
    d = _defines()
    assert d["SD_OK"] == 0
    for code, name in binding.SD_ERR.items():
        assert d[name] == code and code < 0
    assert d["SD_DRAFT_AFTER_ACCEPT"] == 0 and d["SD_DRAFT_ALL_NODES"] == 1
    assert d["SD_LABELS_KEEP_BASE"] == 0 and d["SD_LABELS_KEEP_ALL"] == 1


def test_version_and_kv_bytes_are_host_only(lib):
    assert lib.sd_version().decode().startswith("libspecdec")
    cfg = binding._Config(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32016, n_medusa=4,
                          topk=10, dtype=1, trunc_fallback=0, rope_theta=1e6, rms_eps=1e-5)
    # layers * (K and V) * batch * heads * rows rounded up to blocks of 32 * head_dim * 2 bytes
    assert lib.sd_kv_bytes(C.byref(cfg), 1, 2048) == 32 * 2 * 1 * 32 * 2048 * 128 * 2
    assert lib.sd_kv_bytes(C.byref(cfg), 8, 4097) == 32 * 2 * 8 * 32 * 4128 * 128 * 2
    assert lib.sd_kv_bytes(None, 1, 16) == 0 and lib.sd_kv_bytes(C.byref(cfg), 0, 16) == 0


def test_null_arguments_are_refused_before_any_device_call(lib):
    d = _defines()
    null = None
    assert lib.sd_spec_step(null, null, null, null, null, null) == d["SD_ERR_NULL"]
    assert b"NULL" in lib.sd_last_error()
    assert lib.sd_greedy_step(null, null, null, null) == d["SD_ERR_NULL"]
    assert lib.sd_prefill(null, null, null, null, null) == d["SD_ERR_NULL"]
    assert lib.sd_kv_commit_rows(null, null, null, null, 4, null) == d["SD_ERR_NULL"]
    assert lib.sd_set_draft_schedule(null, 0) == d["SD_ERR_NULL"]
    assert lib.sd_set_graph_mode(null, 1) == d["SD_ERR_NULL"]
    assert lib.sd_set_greedy_drafts(null, 1) == d["SD_ERR_NULL"]
    assert lib.sd_set_fused(null, 1) == d["SD_ERR_NULL"]
    assert lib.sd_set_sync_timeout(null, 5) == d["SD_ERR_NULL"]
    assert lib.sd_set_layer_timeline(null, null, 0) == d["SD_ERR_NULL"]
    assert lib.sd_profile_begin(null, 16) == d["SD_ERR_NULL"]
    assert lib.sd_model_create(null, null, 64, null, null) == d["SD_ERR_NULL"]
    # destroying nothing is allowed
    assert lib.sd_model_destroy(null) == 0 and lib.sd_kv_destroy(null) == 0 and lib.sd_tree_destroy(null) == 0


def _i32(values):
    return (C.c_int32 * len(values))(*values)


@pytest.mark.parametrize("parent,depth,rank,why", [
    ([0, 0], [0, 1], [0, 0], b"root"),                       # node 0 is not a root
    ([-1, 1], [0, 1], [0, 0], b"parent must precede"),       # a node that is its own parent
    ([-1, 0, 0], [0, 1, 2], [0, 0, 1], b"depth"),            # depth not parent's + 1
    ([-1, 0, 1, 2], [0, 1, 2, 3], [0, 0, 0, 0], b"exceeds"), # deeper than the two heads
    ([-1, 0, 0], [0, 1, 1], [0, 4, 1], b"rank"),             # rank >= top-k
    ([-1, 0, 0], [0, 1, 1], [0, 1, 1], b"siblings"),         # two children with the same candidate
])
def test_malformed_trees_are_refused_on_the_host(lib, parent, depth, rank, why):
    d = _defines()
    out = C.c_void_p()
    rc = lib.sd_tree_create(len(parent), _i32(parent), _i32(depth), _i32(rank), 2, 4, C.byref(out))
    assert rc == d["SD_ERR_BAD_TREE"] and not out.value
    assert why in lib.sd_last_error()


def test_tree_size_limits(lib):
    d = _defines()
    out = C.c_void_p()
    assert lib.sd_tree_create(0, _i32([-1]), _i32([0]), _i32([0]), 2, 4, C.byref(out)) == d["SD_ERR_BAD_TREE"]
    n = 257
    assert lib.sd_tree_create(n, _i32([-1] + [0] * (n - 1)), _i32([0] + [1] * (n - 1)), _i32(list(range(n))), 2, 1000,
                              C.byref(out)) == d["SD_ERR_BAD_TREE"]
    assert lib.sd_tree_create(1, None, None, None, 2, 4, C.byref(out)) == d["SD_ERR_NULL"]


def test_bad_configurations_are_refused_before_allocation(lib):
    d = _defines()
    good = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024, n_medusa=3, topk=4, dtype=1,
                trunc_fallback=0, rope_theta=1e4, rms_eps=1e-5)
    one = (C.c_void_p * 4)(1, 1, 1, 1)
    ptrs = C.cast(one, C.POINTER(C.c_void_p))
    w = binding._Weights(1, 1, 1, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs)
    out = C.c_void_p()
    for bad in (dict(dtype=2), dict(head_dim=96, d_model=384), dict(d_model=260), dict(d_ffn=100), dict(n_medusa=16),
                dict(topk=33), dict(topk=0), dict(vocab=1), dict(trunc_fallback=5), dict(rope_theta=0.0)):
        cfg = binding._Config(**{**good, **bad})
        assert lib.sd_model_create(C.byref(cfg), C.byref(w), 64, None, C.byref(out)) == d["SD_ERR_SHAPE"], bad
        assert not out.value
    cfg = binding._Config(**good)
    # cache sizes: bf16 rows in blocks of 32, float32 rows as they are
    assert lib.sd_kv_bytes(C.byref(cfg), 2, 100) == 2 * 2 * 2 * 128 * 256 * 2
    assert lib.sd_kv_bytes(C.byref(binding._Config(**{**good, "dtype": 0})), 2, 100) == 2 * 2 * 2 * 100 * 256 * 4
    assert lib.sd_model_create(C.byref(cfg), C.byref(w), 0, None, C.byref(out)) == d["SD_ERR_SHAPE"]
    assert lib.sd_model_create(C.byref(cfg), C.byref(w), 257, None, C.byref(out)) == d["SD_ERR_SHAPE"]


def test_label_and_sampling_argument_checks(lib):
    d = _defines()
    assert lib.sd_build_labels(None, 0, 16, 2, 5, 6, -100, 0, None, None) == d["SD_ERR_SHAPE"]        # batch
    assert lib.sd_build_labels(None, 1, 16, 65, 5, 6, -100, 0, None, None) == d["SD_ERR_SHAPE"]       # heads
    assert lib.sd_build_labels(None, 1, 16, 2, 5, 6, -100, 7, None, None) == d["SD_ERR_SHAPE"]        # policy
    assert lib.sd_build_labels(None, 1, 0, 2, 5, 6, -100, 0, None, None) == 0                          # empty: nothing to do
    assert lib.sd_build_labels(None, 1, 16, 2, 5, 6, -100, 0, None, None) == d["SD_ERR_NULL"]
