"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every function the
header declares, and its host-side argument validation behaves as documented."""
import os
import re

import pytest

from paper_2603_03333_amd import binding as dmb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "dropmatch.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"^(?:dm_status|const char\*|int32_t)\s+(\w+)\s*\(", src, flags=re.M)
    assert "dropmatch_verify" in names and "dm_create" in names
    return names


def test_library_exports_every_declared_function():
    lib = dmb.load_library()
    declared = _declared_functions()
    assert sorted(declared) == sorted(dmb.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_params_struct_matches_header_field_order():
    src = open(os.path.join(ROOT, "include", "dropmatch.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} dm_params;", src, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = [re.findall(r"(\w+)\s*$", decl.strip())[0] for decl in body.split(";") if decl.strip()]
    assert fields == [f[0] for f in dmb.dm_params._fields_]


def _prm(**kw):
    base = dict(B=1, T=5, K=8, d=256, V=4096, dtype=dmb.DM_F32, p=0.1, seeds=[0])
    base.update(kw)
    parent_ptr = base.pop("parent_ptr", None)
    prm, keep = dmb.make_params(**base)
    if parent_ptr is not None:
        prm.parent = parent_ptr      # never dereferenced by dm_validate
    return prm, keep


def test_validate_accepts_the_benchmark_shapes():
    for kw in (dict(), dict(d=4096, V=128256, dtype=dmb.DM_BF16, T=8, K=16),
               dict(d=8192, V=128256, dtype=dmb.DM_BF16, B=32, T=8, K=16, seeds=list(range(32))),
               dict(d=4096, V=151936, dtype=dmb.DM_BF16, B=4, T=8, K=32, p=0.2, seeds=[1, 2, 3, 4]),
               dict(p=0.0), dict(rule=dmb.DM_RULE_MAJORITY, flags=dmb.DM_FLAG_SHARE_MASK_ACROSS_POS),
               dict(rule=dmb.DM_RULE_JS, K=5, p=0.3), dict(rule=dmb.DM_RULE_JS_OR_MAJORITY, K=64),
               dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=0.7, top_p=0.9, K=64),
               dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=0.7, top_p=1.0, K=200), dict(top_p=7.0)):
        prm, keep = _prm(**kw)
        assert dmb.dm_validate(prm) == (dmb.DM_OK, "")


@pytest.mark.parametrize("kw,word", [
    (dict(B=0), "B"), (dict(T=0), "T"), (dict(T=5000), "T"), (dict(K=0), "K"), (dict(K=2000), "K"),
    (dict(T=4096, K=8), "T*K"), (dict(d=0), "d"), (dict(V=0), "V"), (dict(dtype=7), "dtype"),
    (dict(p=1.0), "p"), (dict(p=-0.5), "p"), (dict(p=float("nan")), "p"), (dict(rule=4), "rule"), (dict(rule=-1), "rule"),
    (dict(rule=dmb.DM_RULE_JS, K=65), "K <= 64"), (dict(rule=dmb.DM_RULE_JS_OR_MAJORITY, parent_ptr=1), "chains"),
    (dict(flags=64), "flags"), (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS), "temperature"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=float("inf")), "temperature"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, rule=dmb.DM_RULE_JS), "token-level"), (dict(flags=dmb.DM_FLAG_CLEAN_LAST_PATH, K=1), "K >= 2"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=1.5), "top_p"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=-0.1), "top_p"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=float("nan")), "top_p"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=0.9, K=65), "K <= 64"),
    (dict(flags=dmb.DM_FLAG_SAMPLE_PATHS, temperature=1.0, top_p=0.9, T=1024, K=16), "T*K"),
])
def test_validate_rejects(kw, word):
    prm, keep = _prm(**kw)
    st, msg = dmb.dm_validate(prm)
    assert st == dmb.DM_EINVAL and word in msg


def test_validate_rejects_null_seeds_and_null_params():
    prm, keep = _prm()
    prm.seeds = None
    st, msg = dmb.dm_validate(prm)
    assert st == dmb.DM_EINVAL and "seeds" in msg
    assert dmb.load_library().dm_validate(None, None, 0) == dmb.DM_EINVAL


def test_kernel_choice():
    assert dmb.dm_kernel_choice(_prm()[0]) == 0                                        # fp32 -> generic
    assert dmb.dm_kernel_choice(_prm(dtype=dmb.DM_BF16, d=4096)[0]) == 1               # bf16, d % 64 == 0
    assert dmb.dm_kernel_choice(_prm(dtype=dmb.DM_BF16, d=100)[0]) == 0
    assert dmb.dm_kernel_choice(_prm(dtype=dmb.DM_BF16, d=4096, flags=dmb.DM_FLAG_FORCE_GENERIC)[0]) == 0
    assert dmb.dm_kernel_choice(_prm(K=0)[0]) == dmb.DM_EINVAL


def test_create_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(dmb.DropMatchError) as ei:
        dmb.dm_create(0, 128, 256, 4096)
    assert ei.value.status == dmb.DM_EHIP and ei.value.message
    import ctypes
    prm, keep = _prm()
    st = dmb.load_library().dropmatch_verify(None, ctypes.byref(prm), *([None] * 11))
    assert st == dmb.DM_EINVAL and "ctx" in dmb.dm_last_error(None)


def test_tree_inputs_for_a_vocabulary_smaller_than_a_sibling_group():
    """The seeded tree generator keeps siblings distinct only while the vocabulary allows it
    (with V = 1 every node carries token 0)."""
    import numpy as np
    from paper_2603_03333_amd import workloads as wk
    wl = wk.Workload("t", d=8, V=1, dtype="f32", B=2, T=9, K=2, p=0.1, tree=True, data_seed=5)
    parent = wk.make_tree_parents(wl, max_depth=4, max_branch=3)
    ids = wk.make_tree_draft_ids(wl, parent, greedy=np.zeros((2, 9), dtype=np.int32))
    assert (ids[:, 0] == -1).all() and (ids[:, 1:] == 0).all()
    assert (parent[:, 1:] < np.arange(1, 9)[None, :]).all() and (parent[:, 0] == -1).all()


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with a plain C compiler, warnings on,
    and every declared function must be usable from C (address taken, nothing linked)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = open(os.path.join(ROOT, "include", "dropmatch.h")).read()
    names = sorted(set(re.findall(r"\b(dm_[a-z_]+|dropmatch_[a-z_]+)\s*\(", src)) & set(dmb.EXPORTS))
    assert names == sorted(dmb.EXPORTS)
    c = tmp_path / "use_header.c"
    c.write_text('#include "dropmatch.h"\n#include <stddef.h>\n'
                 "int main(void) {\n  dm_params p;\n  const void* f[] = {" +
                 ", ".join(f"(const void*)(size_t)&{n}" for n in names) +
                 "};\n  p.top_p = 0.0f; p.temperature = 0.0f;\n  return (int)(sizeof f / sizeof f[0]) * 0 + (int)p.top_p;\n}\n")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(c)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
