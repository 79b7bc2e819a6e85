"""CPU checks of the host side: the built library exports what the header declares, and the
block layouts of the binding agree with Eq. 2 / Eq. 3 as the oracle evaluates them."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import space_oracle as so
from paper_2402_11809_amd import binding, layout as lo
from tests import gpu_common as gc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "space.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(space_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.library_path()):
        from paper_2402_11809_amd.build import build
        build(verbose=False)
    lib = ctypes.CDLL(binding.library_path())
    declared = _declared_symbols()
    assert set(declared) == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_binding_structs_match_header_field_order():
    text = open(os.path.join(ROOT, "include", "space.h")).read()
    for struct, cls in (("space_config", binding.SpaceConfig), ("space_kv", binding.SpaceKV),
                        ("space_step_out", binding.SpaceStepOut), ("space_layer_weights", binding.SpaceLayerWeights),
                        ("space_weights", binding.SpaceWeights)):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (struct, struct), text, flags=re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        names = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            for part in decl.split(","):
                names.append(re.findall(r"(\w+)\s*$", part.strip())[0])
        assert names == [f[0] for f in cls._fields_], struct


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_paper_layout_matches_eq2_eq3(k):
    spec = lo.paper_layout(k)
    toks, is_mask = so.extended_input([7], list(range(k)), k, mask_id=-1)
    assert spec.n_rows == (k + 1) ** 2 == len(toks)
    assert np.array_equal(spec.is_mask.astype(bool), is_mask)
    A = so.sar_attention_mask(is_mask, k)
    assert np.array_equal(gc.rel_pos(spec), so.position_ids(A))
    # the in-block visibility rule the kernels apply, evaluated on the host
    vis = np.zeros_like(A)
    for i in range(spec.n_rows):
        for j in range(i + 1):
            if not spec.is_mask[j] or (spec.is_mask[i] and spec.group[i] == spec.group[j]):
                vis[i, j] = 1
    assert np.array_equal(vis, A)
    assert gc.real_rows(spec) == [g * (k + 1) for g in range(k + 1)]


def test_other_layouts():
    f = lo.first_step_layout(4)
    assert list(f.is_mask) == [0, 1, 1, 1, 1] and list(gc.rel_pos(f)) == [0, 1, 2, 3, 4]
    p = lo.prefill_layout(5)
    assert p.n_groups == 5 and list(gc.rel_pos(p)) == [0, 1, 2, 3, 4]
    g = lo.grouped_layout(4, 7)
    assert g.n_rows == 32 and g.n_groups == 4


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_page_allocator():
    from paper_2402_11809_amd.serving import PageAllocator, pages_for
    a = PageAllocator(5)
    assert a.n_free == 5 and pages_for(0) == 0 and pages_for(1) == 1 and pages_for(32) == 1 and pages_for(33) == 2
    p = a.alloc(3)
    assert sorted(p) == sorted(set(p)) and len(p) == 3 and a.n_free == 2
    assert a.alloc(3) is None and a.n_free == 2          # all or nothing
    q = a.alloc(2)
    assert not set(p) & set(q) and a.n_free == 0 and a.alloc(0) == []
    a.free(p[:1])
    assert a.n_free == 1
    with pytest.raises(ValueError):
        a.free(p[:1])                                     # double free
    with pytest.raises(ValueError):
        a.free([7])
    a.free(p[1:] + q)
    assert a.n_free == 5 and sorted(a.alloc(5)) == [0, 1, 2, 3, 4]


def test_header_is_plain_c_and_structs_have_the_bound_sizes(tmp_path):
    """include/space.h must compile as C99 on its own (the boundary has no C++ or torch types), and the
    ctypes mirrors must have the sizes the C compiler gives the structs."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    from paper_2402_11809_amd import binding
    structs = {"space_config": binding.SpaceConfig, "space_kv": binding.SpaceKV, "space_step_out": binding.SpaceStepOut,
               "space_sample_io": binding.SpaceSampleIO, "space_sample_params": binding.SpaceSampleParams,
               "space_layer_weights": binding.SpaceLayerWeights, "space_weights": binding.SpaceWeights}
    src = tmp_path / "sizes.c"
    lines = ['#include "space.h"', "#include <stdio.h>", "int main(void) {"]
    lines += [f'    printf("{name} %zu\\n", sizeof({name}));' for name in structs]
    lines += ["    return 0;", "}"]
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "sizes"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    sizes = dict(zip(out[::2], (int(v) for v in out[1::2])))
    import ctypes
    for name, cls in structs.items():
        assert sizes[name] == ctypes.sizeof(cls), name


def test_sar_transform_matches_oracle():
    """space_sar_transform (host function of the library; Methods, "Semi-Autoregressive Finetuning") against
    the oracle's dataloader transform on seeded samples: same inputs, same labels, same position."""
    from oracle import space_sft as sf
    rng = np.random.default_rng(12)
    n_sar = 0
    for case in range(200):
        k = int(rng.integers(1, 7))
        n_prompt, n_answer = int(rng.integers(1, 9)), int(rng.integers(k + 1, 40))
        toks = [int(t) for t in rng.integers(0, 1000, size=n_prompt + n_answer)]
        p_ar = float(np.float32(rng.choice([0.0, 0.3, 0.5, 1.0])))
        u_keep, u_pos = float(np.float32(rng.uniform())), float(np.float32(rng.uniform(0, 0.999)))
        ids, labels, m = binding.sar_transform(toks, n_prompt, k, 1000, p_ar, u_keep, u_pos)
        ref = sf.sar_transform(toks[:n_prompt], toks[n_prompt:], k, 1000, p_ar, u_keep, u_pos)
        assert ids == ref.input_ids and labels == ref.labels and m == (ref.m or 0), case
        n_sar += m > 0
    assert 40 < n_sar < 160
    with pytest.raises(binding.SpaceError) as e:
        binding.sar_transform([1, 2, 3, 4], 1, 3, 9, 0.0, 0.5, 0.5)   # answer of 3 tokens, k = 3
    assert e.value.code == binding.SPACE_ESHAPE
