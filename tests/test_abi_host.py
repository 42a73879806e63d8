"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares, and the plan
validates shapes and lays out buffers without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def llsa():
    from paper_2512_16615_amd import build, llsa as binding
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    binding.load()
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "llsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(llsa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(llsa):
    lib = ctypes.CDLL(llsa.LIB_PATH)
    names = _declared_functions()
    assert "llsa_forward" in names and "llsa_backward" in names and "llsa_plan" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(llsa.EXPORTS) == names


def test_plan_level_table_headline(llsa):
    p = llsa.Plan(1, 16, 65536, 64, 16, 8, 3)
    assert [(li.rows, li.K_l) for li in p.levels] == [(4096, 8), (256, 8), (16, 8)]
    assert p.indices_bytes() == 16 * (4096 + 256 + 16) * 8 * 4
    pooled = 3 * 16 * (4096 + 256 + 16) * 64 * 2
    assert pooled <= p.workspace_bytes(False) <= pooled + 9 * 256
    assert p.workspace_bytes(True) > p.workspace_bytes(False)
    for x in range(3):
        assert p.pyramid_info(x, 1)[0] == 4096 and p.pyramid_info(x, 3)[0] == 16


def test_plan_other_block_sizes_and_wide_lists(llsa):
    p = llsa.Plan(1, 16, 65536, 64, 64, 8, 2)           # B = 64: 65536 -> 1024 -> 16
    assert [(li.rows, li.K_l) for li in p.levels] == [(1024, 8), (16, 8)]
    pooled = 3 * 16 * (1024 + 16) * 64 * 2
    assert pooled <= p.workspace_bytes(False) <= pooled + 6 * 256
    p = llsa.Plan(1, 2, 32768, 64, 32, 4, 3)            # B = 32: 32768 -> 1024 -> 32 -> 1
    assert [(li.rows, li.K_l) for li in p.levels] == [(1024, 4), (32, 4), (1, 1)]
    p = llsa.Plan(1, 2, 65536, 64, 16, 64, 3)           # K = 64: capped by the rows of the level above
    assert [(li.rows, li.K_l) for li in p.levels] == [(4096, 64), (256, 64), (16, 16)]
    assert p.indices_bytes() == 2 * (4096 * 64 + 256 * 64 + 16 * 16) * 4
    with pytest.raises(llsa.LlsaError):
        llsa.Plan(1, 2, 65536, 64, 16, 65, 3)           # K beyond 64


def test_plan_partial_top_level(llsa):
    p = llsa.Plan(2, 16, 16384, 64, 16, 8, 3)          # top level holds 4 tokens: K_2 = 4
    assert [(li.rows, li.K_l) for li in p.levels] == [(1024, 8), (64, 8), (4, 4)]
    p = llsa.Plan(1, 1, 256, 32, 4, 2, 3, dtype=llsa.F32)
    assert [(li.rows, li.K_l) for li in p.levels] == [(64, 2), (16, 2), (4, 2)]


@pytest.mark.parametrize("kw,status", [
    (dict(N=65536 + 16), 2),          # not divisible by B^L
    (dict(L=0), 2),
    (dict(Le=4), 2),
    (dict(K=0), 2),
    (dict(d=48), 3),
    (dict(dtype=7), 3),
    (dict(B=128), 3),
    (dict(L=1), 3),                    # 4096 coarse tokens: fine;  see below
    (dict(N=262144, L=1, kernel_path=1), 3),   # 16384 candidates per row: beyond the portable selection's LDS row
])
def test_plan_rejects_bad_problems(llsa, kw, status):
    args = dict(batch=1, heads=16, N=65536, d=64, B=16, K=8, L=3, Le=None)
    args.update(kw)
    if kw == dict(L=1):
        llsa.Plan(**args)             # single-level selection over 4096 coarse tokens is supported
        return
    with pytest.raises(llsa.LlsaError) as e:
        llsa.Plan(**args)
    assert f"status {status}" in str(e.value)
    if "kernel_path" in kw:             # the chunked selection of the MFMA path takes any number of candidates
        del args["kernel_path"]
        llsa.Plan(**args)


def test_null_pointers_are_refused_before_any_launch(llsa):
    p = llsa.Plan(1, 1, 256, 32, 4, 2, 3, dtype=llsa.F32)
    lib = llsa.load()
    assert lib.llsa_forward(p._h, None, None, None, None, None, None, None, None) == 1
    assert lib.llsa_backward(p._h, *([None] * 12)) == 1
    assert lib.llsa_plan(None, None) == 1
    assert lib.llsa_status_string(0) == b"ok"


def test_desc_layout_matches_the_header(llsa):
    """The binding's struct must list the header's fields in the header's order (same C layout)."""
    text = open(os.path.join(ROOT, "include", "llsa.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} llsa_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            names += [n.strip() for n in decl.split(None, 1)[1].split(",")]
    assert names == [f[0] for f in llsa._Desc._fields_]


def test_reorder_validates_on_the_host(llsa):
    """llsa_reorder refuses bad calls before anything is enqueued (no GPU needed to see that)."""
    lib = llsa.load()
    a, b = ctypes.c_void_p(4096), ctypes.c_void_p(1 << 30)       # never dereferenced: every call below is refused
    assert lib.llsa_reorder(1, 4096, 64, llsa.BF16, 0, None, b, None) == 1
    assert lib.llsa_reorder(1, 2048, 64, llsa.BF16, 0, a, b, None) == 2     # not a power of four
    assert lib.llsa_reorder(1, 4096, 4, llsa.BF16, 0, a, b, None) == 2      # 8-byte rows
    assert lib.llsa_reorder(1, 4096, 64, 9, 0, a, b, None) == 3             # unknown dtype
    assert lib.llsa_reorder(1, 4096, 64, llsa.BF16, 0, a, ctypes.c_void_p(4096 + 128), None) == 2   # overlap


def test_forward_static_checks_the_size_on_the_host(llsa):
    """llsa_forward_static refuses NULL and a plan beyond the static workspace before any HIP call."""
    lib = llsa.load()
    assert lib.llsa_static_workspace_bytes() == 32 << 20
    big = llsa.Plan(1, 8, 262144, 128, 16, 16, 4)                 # pooled levels: about 102 MiB
    assert big.workspace_bytes(False) > lib.llsa_static_workspace_bytes()
    a = ctypes.c_void_p(4096)                                      # never dereferenced
    assert lib.llsa_forward_static(big._h, a, a, a, a, a, a, None) == 4
    assert lib.llsa_forward_static(big._h, a, a, None, a, a, a, None) == 1
    headline = llsa.Plan(1, 16, 65536, 64, 16, 8, 3)
    assert headline.workspace_bytes(False) <= lib.llsa_static_workspace_bytes()


def test_glue_entry_points_and_alignment_are_checked_on_the_host(llsa):
    """NULL, a negative eps and misaligned pointers are refused before any launch, by every compute entry point."""
    lib = llsa.load()
    plan = llsa.Plan(1, 3, 4096, 64, 16, 8, 2)
    a, odd = ctypes.c_void_p(4096), ctypes.c_void_p(4100)
    eps = ctypes.c_float(1e-6)
    assert lib.llsa_qknorm_rope_pool(plan._h, None, a, a, a, a, a, a, eps, a, a, a, None) == 1
    assert lib.llsa_qknorm_rope_pool(plan._h, a, a, a, a, a, a, a, ctypes.c_float(-1.0), a, a, a, None) == 2
    assert lib.llsa_qknorm_rope_pool(plan._h, odd, a, a, a, a, a, a, eps, a, a, a, None) == 2
    assert lib.llsa_forward_pooled(plan._h, a, a, a, a, a, a, None, None) == 1
    assert lib.llsa_forward(plan._h, a, odd, a, a, a, a, a, None) == 2
    assert lib.llsa_forward(plan._h, a, a, a, a, a, a, ctypes.c_void_p(4096 + 16), None) == 2     # workspace: 256 bytes
    assert lib.llsa_backward(plan._h, a, a, a, a, a, a, a, a, a, odd, a, None) == 2
    assert lib.llsa_attention(plan._h, a, a, a, a, a, odd, a, None) == 2
    assert lib.llsa_pool(plan._h, a, a, odd, a, None) == 2


def test_plan_refuses_sizes_beyond_32_bit_grids(llsa):
    """Launch grids and the key-major list offsets are 32-bit: a plan that would overflow them is refused."""
    with pytest.raises(llsa.LlsaError) as e:
        llsa.Plan(1 << 10, 1 << 10, 1 << 20, 64, 16, 8, 4)          # 2^20 heads x 2^16 tiles
    assert "status 3" in str(e.value)
    llsa.Plan(1, 4, 1 << 20, 64, 16, 8, 4)                           # the largest tested shape is fine
