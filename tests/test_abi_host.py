"""Host-side checks of the C ABI: the library loads, exports what the header declares,
and rejects bad arguments before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2504_14051_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2504_14051_amd import build
        build.build()
    binding.lib()
    return binding


def good_layout(B, **kw):
    d = kw.pop("head_dim", 128)
    cap = kw.pop("capacity", 1024)
    W = kw.pop("window", 8)
    hq, hkv = kw.pop("n_q_heads", 8), kw.pop("n_kv_heads", 2)
    L = B.Layout(batch=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, window=W, capacity=cap,
                 seq_lens=None,
                 k_stride_b=hkv * cap * d, k_stride_h=cap * d, k_stride_n=d,
                 v_stride_b=hkv * cap * d, v_stride_h=cap * d, v_stride_n=d,
                 q_stride_b=hq * W * d, q_stride_h=W * d, q_stride_w=d,
                 dtype=B.BF16, base=B.BASE_H2O, softmax_scale=0.088, pool_kernel=1,
                 window_in_cache=1, n_protect_head=0, n_protect_tail=0, variant=B.EXACT)
    for k, v in kw.items():
        setattr(L, k, v)
    return L


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "caote.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(caote_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in caote.h but not exported"
    assert B.caote_version() >= 100


def test_layout_struct_matches_header_field_order(B):
    header = open(os.path.join(ROOT, "include", "caote.h")).read()
    body = re.search(r"typedef struct caote_layout \{(.*?)\} caote_layout;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        decl = re.sub(r"^(const\s+)?(int32_t|int64_t|float)\s*\*?", "", decl)
        names += [n.strip() for n in decl.split(",")]
    assert names == [f[0] for f in B.Layout._fields_]


def test_workspace_bytes_positive_and_monotone_in_budget(B):
    L = good_layout(B)
    w0 = B.caote_workspace_bytes(L, 0)
    w1 = B.caote_workspace_bytes(L, 256)
    assert 0 < w0 <= w1
    assert w0 % 256 == 0


@pytest.mark.parametrize("field,value,status", [
    ("head_dim", 96, "EUNSUPPORTED"), ("n_q_heads", 7, "EINVAL"), ("window", 0, "EINVAL"),
    ("capacity", 0, "EINVAL"), ("pool_kernel", 4, "EINVAL"), ("pool_kernel", 0, "EINVAL"),
    ("dtype", 5, "EINVAL"), ("base", 3, "EINVAL"), ("variant", 2, "EINVAL"),
    ("k_stride_n", 132, "EINVAL"), ("k_stride_n", 64, "EINVAL"), ("n_protect_tail", -1, "EINVAL"),
    ("softmax_scale", float("nan"), "EINVAL"), ("window", 2048, "EINVAL"), ("batch", 0, "EINVAL"),
])
def test_bad_layout_is_rejected_on_the_host(B, field, value, status):
    L = good_layout(B)
    setattr(L, field, value)
    with pytest.raises(B.CaoteError) as e:
        B.caote_workspace_bytes(L, 16)
    fake = 0x1000   # never dereferenced: validation fails first
    with pytest.raises(B.CaoteError) as e:
        B.caote_score(fake, fake, fake, fake, L, fake, fake, stream=0, workspace_bytes=1 << 30)
    assert e.value.status == getattr(B, status)
    assert B.caote_last_error() != ""


def test_null_pointers_budget_mode_and_workspace_errors(B):
    L = good_layout(B)
    fake, ws = 0x1000, 0x10000
    need = B.caote_workspace_bytes(L, 64)
    with pytest.raises(B.CaoteError) as e:                       # null K
        B.caote_score(fake, None, fake, fake, L, fake, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:                       # H2O without an accumulator
        B.caote_score(fake, fake, fake, None, L, fake, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL and "H2O" in str(e.value)
    with pytest.raises(B.CaoteError) as e:                       # budget < 1
        B.caote_select(fake, L, 0, fake, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:                       # bad mode
        B.caote_compact(fake, fake, None, fake, L, 64, 7, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL
    big = good_layout(B, capacity=40000)                         # hole-filling mode: budget limit
    with pytest.raises(B.CaoteError) as e:
        B.caote_compact(fake, fake, None, fake, big, B.FILL_MAX_BUDGET + 1, B.COMPACT_FILL, ws, stream=0,
                        workspace_bytes=B.caote_workspace_bytes(big, B.FILL_MAX_BUDGET + 1))
    assert e.value.status == B.EUNSUPPORTED and "CAOTE_COMPACT_FILL" in str(e.value)
    with pytest.raises(B.CaoteError) as e:
        B.caote_evict(fake, fake, fake, fake, big, B.FILL_MAX_BUDGET + 1, B.COMPACT_FILL, fake, fake, ws, stream=0,
                      workspace_bytes=B.caote_workspace_bytes(big, B.FILL_MAX_BUDGET + 1))
    assert e.value.status == B.EUNSUPPORTED
    with pytest.raises(B.CaoteError) as e:                       # workspace too small
        B.caote_select(fake, L, 64, fake, ws, stream=0, workspace_bytes=need - 1)
    assert e.value.status == B.EWORKSPACE and "needed" in str(e.value)
    with pytest.raises(B.CaoteError) as e:                       # workspace NULL
        B.caote_select(fake, L, 64, fake, None, stream=0, workspace_bytes=need)
    assert e.value.status == B.EWORKSPACE
    with pytest.raises(B.CaoteError) as e:                       # workspace misaligned
        B.caote_select(fake, L, 64, fake, ws + 8, stream=0, workspace_bytes=need)
    assert e.value.status == B.EWORKSPACE
    with pytest.raises(B.CaoteError) as e:                       # evict: null kept_idx
        B.caote_evict(fake, fake, fake, fake, L, 64, 0, fake, None, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2504_14051_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libcaote_hip.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.lib()


def test_append_arguments_are_checked_on_the_host(B):
    L = good_layout(B)
    fake = 0x1000
    with pytest.raises(B.CaoteError) as e:                       # rows do not fit
        B.caote_append(fake, fake, None, fake, fake, L, L.capacity - 3, 4, stream=0)
    assert e.value.status == B.EINVAL and "capacity" in str(e.value)
    with pytest.raises(B.CaoteError) as e:                       # null source
        B.caote_append(fake, fake, None, None, fake, L, 0, 4, stream=0)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:                       # misaligned source
        B.caote_append(fake, fake, None, fake + 8, fake, L, 0, 4, stream=0)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:
        B.caote_append(fake, fake, None, fake, fake, L, 0, -1, stream=0)
    assert e.value.status == B.EINVAL
    B.caote_append(fake, fake, None, fake, fake, L, 0, 0, stream=0)   # nothing to do: no launch


def test_joint_eviction_arguments_are_checked_on_the_host(B):
    fake = 0x1000

    def call(L, budget, evicted=fake, err=fake):
        B.caote_evict_joint(fake, fake, fake, fake, L, budget, 0, fake, fake, evicted, err, fake,
                            stream=0, workspace_bytes=1 << 40)

    with pytest.raises(B.CaoteError) as e:                       # beyond the capacity limit
        call(good_layout(B, capacity=B.JOINT_MAX_CAPACITY + 1), 100)
    assert e.value.status == B.EUNSUPPORTED and str(B.JOINT_MAX_CAPACITY) in str(e.value)
    with pytest.raises(B.CaoteError) as e:                       # defined for the exact score only
        call(good_layout(B, variant=B.FAST), 100)
    assert e.value.status == B.EUNSUPPORTED
    with pytest.raises(B.CaoteError) as e:                       # fewer slots than protected rows
        call(good_layout(B, n_protect_head=60, n_protect_tail=50), 100)
    assert e.value.status == B.EINVAL and "protected" in str(e.value)
    with pytest.raises(B.CaoteError) as e:                       # outputs missing
        call(good_layout(B), 100, evicted=None)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:
        call(good_layout(B), 100, err=None)
    assert e.value.status == B.EINVAL
    # the header's limit is the binding's
    hdr = open(os.path.join(ROOT, "include", "caote.h")).read()
    assert int(re.search(r"#define\s+CAOTE_JOINT_MAX_CAPACITY\s+(\d+)", hdr).group(1)) == B.JOINT_MAX_CAPACITY


def test_read_stream_arguments_are_checked_on_the_host(B):
    fake = 0x1000
    for args in ((None, 16, fake), (fake, 16, None), (fake + 4, 16, fake), (fake, 20, fake)):
        with pytest.raises(B.CaoteError) as e:
            B.caote_read_stream(*args, stream=0)
        assert e.value.status == B.EINVAL
    B.caote_read_stream(fake, 0, fake, stream=0)                 # nothing to read: no launch


def test_issue_probe_arguments_are_checked_on_the_host(B):
    fake = 0x1000
    for variant, iters, out in ((-1, 8, fake), (len(B.ISSUE_PROBE_VARIANTS), 8, fake), (0, 0, fake), (0, 8, None)):
        with pytest.raises(B.CaoteError) as e:
            B.caote_issue_probe(variant, iters, out, stream=0)
        assert e.value.status == B.EINVAL
    hdr = open(os.path.join(ROOT, "include", "caote.h")).read()
    assert int(re.search(r"#define\s+CAOTE_ISSUE_PROBE_VARIANTS\s+(\d+)", hdr).group(1)) == len(B.ISSUE_PROBE_VARIANTS)


def test_misaligned_data_pointers_are_rejected(B):
    """q, K and V are fetched in 16-byte pieces: a base address off that grid is refused on the
    host by every entry point that reads them."""
    L = good_layout(B)
    fake, ws = 0x1000, 0x10000
    need = B.caote_workspace_bytes(L, 64)
    for q, K, V in ((fake + 8, fake, fake), (fake, fake + 2, fake), (fake, fake, fake + 4)):
        with pytest.raises(B.CaoteError) as e:
            B.caote_score(q, K, V, fake, L, fake, ws, stream=0, workspace_bytes=need)
        assert e.value.status == B.EINVAL and "aligned" in str(e.value)
        with pytest.raises(B.CaoteError) as e:
            B.caote_evict(q, K, V, fake, L, 64, 0, fake, fake, ws, stream=0, workspace_bytes=need)
        assert e.value.status == B.EINVAL and "aligned" in str(e.value)
        with pytest.raises(B.CaoteError) as e:
            B.caote_evict_static(q, K, V, fake, L, 64, 0, fake, fake, stream=0)
        assert e.value.status == B.EINVAL and "aligned" in str(e.value)
    with pytest.raises(B.CaoteError) as e:
        B.caote_compact(fake + 8, fake, None, fake, L, 64, 0, ws, stream=0, workspace_bytes=need)
    assert e.value.status == B.EINVAL and "aligned" in str(e.value)
    with pytest.raises(B.CaoteError) as e:
        B.caote_append(fake, fake + 8, None, fake, fake, L, 0, 4, stream=0)
    assert e.value.status == B.EINVAL and "aligned" in str(e.value)


def test_static_scratch_entry_point_checks_arguments_and_size_on_the_host(B):
    """caote_evict_static: the same argument checks as caote_evict, and a layout whose scratch
    does not fit the fixed array is refused before any device call is made."""
    fake = 0x1000
    L = good_layout(B)
    with pytest.raises(B.CaoteError) as e:                       # null kept_idx
        B.caote_evict_static(fake, fake, fake, fake, L, 64, 0, fake, None, stream=0)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:                       # bad mode
        B.caote_evict_static(fake, fake, fake, fake, L, 64, 9, fake, fake, stream=0)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.CaoteError) as e:                       # H2O without an accumulator
        B.caote_evict_static(fake, fake, fake, None, L, 64, 0, fake, fake, stream=0)
    assert e.value.status == B.EINVAL
    big = good_layout(B, capacity=2049, window=1, n_q_heads=32, n_kv_heads=8, batch=16)
    assert B.caote_workspace_bytes(big, 2048) > B.STATIC_SCRATCH_BYTES
    with pytest.raises(B.CaoteError) as e:
        B.caote_evict_static(fake, fake, fake, fake, big, 2048, 1, fake, fake, stream=0)
    assert e.value.status == B.EWORKSPACE and "static" in str(e.value)
    hdr = open(os.path.join(ROOT, "include", "caote.h")).read()
    m = re.search(r"#define\s+CAOTE_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", hdr)
    assert int(m.group(1)) << int(m.group(2)) == B.STATIC_SCRATCH_BYTES
