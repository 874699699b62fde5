"""CPU-only checks of the boundary: the library loads, exports every symbol the header
declares, and its host-only helpers behave.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ecoserve.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2504_18154_amd import build
    build.build()
    from paper_2504_18154_amd import binding as b
    return b


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ecoserve_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(binding):
    names = _declared_symbols()
    assert len(names) >= 14
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ecoserve.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_library_exports_every_symbol_of_the_scheduling_header(binding):
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "ecoserve_padg.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(ecoserve_padg_[a-z0-9_]+)\s*\(", text)))
    assert names == ["ecoserve_padg_check_constraints", "ecoserve_padg_prefill_us", "ecoserve_padg_simulate"]
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ecoserve_padg.h but not exported"


def test_binding_constants_match_the_header(binding):
    """Options, status codes and kernel ids are plain integers on both sides of the boundary."""
    text = open(HEADER).read()
    header = {m.group(1): int(m.group(2)) for m in re.finditer(r"\b(ECOSERVE_[A-Z0-9_]+)\s*=\s*(\d+)", text)}
    mine = {
        "ECOSERVE_OPT_DECODE_SPLIT_TOKENS": binding.OPT_DECODE_SPLIT_TOKENS, "ECOSERVE_OPT_FORCE_PLAIN": binding.OPT_FORCE_PLAIN,
        "ECOSERVE_OPT_PROFILE": binding.OPT_PROFILE, "ECOSERVE_OPT_DECODE_ADAPTIVE": binding.OPT_DECODE_ADAPTIVE,
        "ECOSERVE_OPT_PREFILL_REUSE_PLAN": binding.OPT_PREFILL_REUSE_PLAN,
        "ECOSERVE_OK": binding.OK, "ECOSERVE_EINVAL": binding.EINVAL, "ECOSERVE_ECONTENT": binding.ECONTENT,
        "ECOSERVE_KERNEL_APPEND": binding.KERNEL_APPEND, "ECOSERVE_KERNEL_PREFILL": binding.KERNEL_PREFILL,
        "ECOSERVE_KERNEL_DECODE": binding.KERNEL_DECODE,
    }
    for name, value in mine.items():
        assert header.get(name) == value, f"{name}: header {header.get(name)} vs binding {value}"
    options = {k for k in header if k.startswith("ECOSERVE_OPT_")}
    assert options == {k for k in mine if k.startswith("ECOSERVE_OPT_")}, "an option of the header is missing in the binding"


def test_strerror_and_cache_bytes(binding):
    assert binding.strerror(0) == "ok"
    assert "invalid" in binding.strerror(binding.EINVAL)
    lay = binding.make_layout(40, 8, 128, 1000, "bf16")
    assert binding.cache_bytes(lay) == 1000 * 8 * 16 * 128 * 2
    assert binding.cache_bytes(binding.make_layout(4, 2, 64, 16, "f32")) == 16 * 2 * 16 * 64 * 4
    assert binding.cache_bytes(binding.make_layout(5, 2, 64, 16, "f32")) == 0          # Hq % Hkv != 0
    assert binding.cache_bytes(binding.make_layout(4, 2, 64, 16, "f32", bs=32)) == 0   # block size


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64)])
def test_cache_index_functions_match_logical_views(binding, dtype, D):
    """The C index helpers, the documented layout and the binding's logical views agree:
    fill a CPU 'pool' with its own element offsets and read it through the views."""
    nb, Hkv, bs = 3, 2, 16
    lay = binding.make_layout(4, Hkv, D, nb, dtype)
    n = nb * Hkv * bs * D
    x = 8 if dtype == "bf16" else 4
    offs = torch.arange(n, dtype=torch.int32)
    k_log = offs.view(nb, Hkv, D // x, bs, x).permute(0, 1, 3, 2, 4).reshape(nb, Hkv, bs, D)
    v_log = offs.view(nb, Hkv, D, bs).permute(0, 1, 3, 2)
    rng = np.random.default_rng(0)
    for _ in range(200):
        blk, g, s, d = rng.integers(nb), rng.integers(Hkv), rng.integers(bs), rng.integers(D)
        assert binding.k_cache_index(lay, blk, g, s, d) == int(k_log[blk, g, s, d])
        assert binding.v_cache_index(lay, blk, g, s, d) == int(v_log[blk, g, s, d])
    # bijections onto [0, n)
    assert sorted(k_log.flatten().tolist()) == list(range(n))


def test_create_rejects_bad_layouts_before_touching_a_device(binding):
    h = ctypes.c_void_p()
    lib = binding._lib
    bad = [
        (binding.make_layout(5, 2, 64, 16, "f32"), binding.EINVAL),
        (binding.make_layout(4, 2, 64, 16, "f32", bs=8), binding.EUNSUPPORTED),
        (binding.make_layout(64, 2, 128, 16, "bf16"), binding.EUNSUPPORTED),   # group of 32
        (binding.make_layout(4, 2, 60, 16, "bf16"), binding.EUNSUPPORTED),     # head size not a multiple of 8
        (binding.make_layout(4, 2, 512, 16, "bf16"), binding.EUNSUPPORTED),
    ]
    for lay, want in bad:
        assert lib.ecoserve_create(ctypes.byref(h), 0, ctypes.byref(lay), 4, 4) == want
        assert not h.value
    ok = binding.make_layout(4, 2, 64, 16, "f32")
    assert lib.ecoserve_create(ctypes.byref(h), 0, ctypes.byref(ok), 0, 4) == binding.EINVAL
    assert lib.ecoserve_create(None, 0, ctypes.byref(ok), 4, 4) == binding.EINVAL
    assert lib.ecoserve_destroy(None) == binding.OK
    if not torch.cuda.is_available():
        # no GPU here: a valid request must fail loudly, never fall back
        assert lib.ecoserve_create(ctypes.byref(h), 0, ctypes.byref(ok), 4, 4) == binding.EHIP


def test_split_merge_identity_in_fp64():
    """The algebra the split-context decode relies on: merging (m, l, acc) of any partition
    of the context reproduces the unsplit softmax-weighted sum."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        n, D = int(rng.integers(2, 300)), 8
        s = rng.normal(size=n) * 4
        V = rng.normal(size=(n, D))
        ref = (np.exp(s - s.max()) / np.exp(s - s.max()).sum()) @ V
        cuts = np.sort(rng.choice(np.arange(1, n), size=min(n - 1, int(rng.integers(1, 8))), replace=False))
        parts = np.split(np.arange(n), cuts)
        m = np.array([s[p].max() for p in parts])
        l = np.array([np.exp(s[p] - s[p].max()).sum() for p in parts])
        acc = np.stack([np.exp(s[p] - s[p].max()) @ V[p] for p in parts])
        M = m.max()
        w = np.exp(m - M)
        out = (acc * w[:, None]).sum(0) / (l * w).sum()
        np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
