"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments with the documented status before touching any device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2507_01438_amd import build
    if build.is_stale():
        build.build()
    from paper_2507_01438_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "elora.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(elora_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTED), declared ^ set(B.EXPORTED)
    for name in declared:
        assert hasattr(B.lib, name), name
    assert B.elora_version() >= 1
    assert B.elora_status_string(0) == "ok" and "unknown" in B.elora_status_string(99)


def test_struct_layouts_match_the_header(B):
    # 5 ints (+4 pad), 4 pointers, pool, 3 pointers, int (+4 pad), pointer, pointer, size_t
    assert ctypes.sizeof(B.elora_linear_desc_t) == 24 + 8 * 4 + 8 + 8 * 3 + 8 + 8 + 8 + 8
    assert ctypes.sizeof(B.elora_plan_t) == 24


FAKE = 0x7F0000000000  # an address that is aligned and never dereferenced by host-side checks


def test_pool_sizes_and_create_validation(B):
    assert B.elora_pool_storage_bytes(0, 16, 8, 4, B.ELORA_BF16) == 0
    assert B.elora_pool_storage_bytes(16, 16, 0, 4, B.ELORA_BF16) == 0
    assert B.elora_pool_storage_bytes(16, 16, 8, 4, 7) == 0
    n = B.elora_pool_storage_bytes(4096, 4096, 16, 64, B.ELORA_BF16)
    assert n >= 64 * (4096 + 4096) * 16 * 2 and n % 256 == 0

    def create(*a):
        with pytest.raises(B.EloraError) as e:
            B.elora_pool_create(*a)
        return e.value.status

    assert create(4096, 4096, 16, 64, B.ELORA_BF16, None, n) == B.ELORA_E_NULL
    assert create(4096, 4096, 16, 64, 5, FAKE, n) == B.ELORA_E_DTYPE
    assert create(-1, 4096, 16, 64, B.ELORA_BF16, FAKE, n) == B.ELORA_E_SHAPE
    assert create(4096, 4096, 999, 64, B.ELORA_BF16, FAKE, n) == B.ELORA_E_RANK
    assert create(4096, 4096, 16, 64, B.ELORA_BF16, FAKE + 64, n) == B.ELORA_E_ALIGN
    assert create(4096, 4096, 16, 64, B.ELORA_BF16, FAKE, n - 1) == B.ELORA_E_STORAGE
    h = B.elora_pool_create(4096, 4096, 16, 64, B.ELORA_BF16, FAKE, n)
    assert B.elora_pool_slot_info(h, 3) == (0, 0.0)
    with pytest.raises(B.EloraError) as e:
        B.elora_pool_slot_info(h, 64)
    assert e.value.status == B.ELORA_E_SLOT
    # load/evict argument checks come before any device work
    for args, want in [((h, -1, 8, 1.0, FAKE, FAKE, 1, 0), B.ELORA_E_SLOT),
                       ((h, 64, 8, 1.0, FAKE, FAKE, 1, 0), B.ELORA_E_SLOT),
                       ((h, 0, 17, 1.0, FAKE, FAKE, 1, 0), B.ELORA_E_RANK),
                       ((h, 0, 0, 1.0, FAKE, FAKE, 1, 0), B.ELORA_E_RANK),
                       ((h, 0, 8, 1.0, None, FAKE, 1, 0), B.ELORA_E_NULL)]:
        assert B.lib.elora_pool_load_adapter(*args) == want
    assert B.lib.elora_pool_evict(h, 5, 0) == B.ELORA_E_NOT_LOADED
    assert B.lib.elora_pool_evict(h, 99, 0) == B.ELORA_E_SLOT
    B.elora_pool_destroy(h)
    assert B.lib.elora_pool_destroy(None) == B.ELORA_E_NULL


def _desc(B, pool=None, **over):
    K, N, T = 4096, 4096, 32
    kw = dict(n_tokens=T, d_in=K, d_out=N, dtype=B.ELORA_BF16, x=FAKE, W=FAKE, y=FAKE, workspace=FAKE,
              workspace_bytes=B.elora_workspace_bytes(T, K, N, 16), pool=pool,
              adapter_idx=FAKE if pool else None)
    kw.update(over)
    return B.make_desc(**kw)


def _plan_status(B, d):
    plan = B.elora_plan_t()
    return B.lib.elora_linear_plan(ctypes.byref(d), ctypes.byref(plan))


def test_linear_descriptor_validation(B):
    n = B.elora_pool_storage_bytes(4096, 4096, 16, 64, B.ELORA_BF16)
    h = B.elora_pool_create(4096, 4096, 16, 64, B.ELORA_BF16, FAKE, n)
    assert _plan_status(B, _desc(B, h)) == B.ELORA_OK
    assert _plan_status(B, _desc(B, h, x=None)) == B.ELORA_E_NULL
    assert _plan_status(B, _desc(B, h, workspace=None)) == B.ELORA_E_NULL
    assert _plan_status(B, _desc(B, h, dtype=3)) == B.ELORA_E_DTYPE
    assert _plan_status(B, _desc(B, h, dtype=B.ELORA_F32)) == B.ELORA_E_DTYPE          # pool is bf16
    assert _plan_status(B, _desc(B, h, wfmt=3)) == B.ELORA_E_DTYPE
    assert _plan_status(B, _desc(B, None, wfmt=B.ELORA_W_INT4_G32, dtype=B.ELORA_F32, w_scales=FAKE)) == B.ELORA_E_DTYPE
    assert _plan_status(B, _desc(B, h, wfmt=B.ELORA_W_INT4_G32)) == B.ELORA_E_NULL      # scales missing
    assert _plan_status(B, _desc(B, h, d_in=2048)) == B.ELORA_E_SHAPE                   # pool says 4096
    assert _plan_status(B, _desc(B, h, n_tokens=-1)) == B.ELORA_E_SHAPE
    assert _plan_status(B, _desc(B, h, y=FAKE + 2)) == B.ELORA_E_ALIGN
    assert _plan_status(B, _desc(B, h, workspace=FAKE + 16)) == B.ELORA_E_ALIGN
    assert _plan_status(B, _desc(B, h, workspace_bytes=1024)) == B.ELORA_E_STORAGE
    assert _plan_status(B, _desc(B, h, adapter_idx=None)) == B.ELORA_E_SEGMENTS         # neither form
    assert _plan_status(B, _desc(B, h, seg_offsets=FAKE, seg_adapter=FAKE, n_segments=2)) == B.ELORA_E_SEGMENTS  # both
    assert _plan_status(B, _desc(B, h, adapter_idx=None, seg_offsets=FAKE)) == B.ELORA_E_SEGMENTS
    assert _plan_status(B, _desc(B, h, adapter_idx=None, seg_offsets=FAKE, seg_adapter=FAKE, n_segments=-1)) == B.ELORA_E_SEGMENTS
    assert _plan_status(B, _desc(B, h, adapter_idx=None, seg_offsets=FAKE, seg_adapter=FAKE, n_segments=3)) == B.ELORA_OK
    assert B.lib.elora_linear_plan(None, ctypes.byref(B.elora_plan_t())) == B.ELORA_E_NULL
    assert B.lib.elora_batched_lora_linear(None, 0) == B.ELORA_E_NULL
    B.elora_pool_destroy(h)


def test_kernel_family_selection(B):
    n = B.elora_pool_storage_bytes(4096, 4096, 16, 64, B.ELORA_BF16)
    h = B.elora_pool_create(4096, 4096, 16, 64, B.ELORA_BF16, FAKE, n)
    p = B.elora_linear_plan(_desc(B, h))
    # (the K-split depends on how many workgroups the device holds at once; without a device the plan is a cautious one)
    assert p.path == B.ELORA_PATH_DECODE and p.n_launches == 1 and p.split_k in (1, 2, 4, 8)
    assert p.grid >= 64 * p.split_k and p.grid % (8 * p.split_k) == 0 and p.tile_rows == 64
    # fp32 and odd shapes go to the plain-ALU kernels
    p = B.elora_linear_plan(_desc(B, None, dtype=B.ELORA_F32, d_in=512, d_out=512, n_tokens=8))
    assert p.path == B.ELORA_PATH_GENERIC
    p = B.elora_linear_plan(_desc(B, None, d_in=100, d_out=30, n_tokens=8))
    assert p.path == B.ELORA_PATH_GENERIC
    B.elora_force_path(B.ELORA_PATH_GENERIC)
    try:
        assert B.elora_linear_plan(_desc(B, h)).path == B.ELORA_PATH_GENERIC
    finally:
        B.elora_force_path(-1)
    with pytest.raises(B.EloraError):
        B.elora_force_path(9)
    assert B.elora_workspace_bytes(32, 4096, 4096, 0) == 0
    B.elora_pool_destroy(h)


def test_workspace_init_and_hooks_validate_arguments(B):
    assert B.lib.elora_workspace_init(None, 1 << 20, 0) == B.ELORA_E_NULL
    assert B.lib.elora_workspace_init(FAKE + 8, 1 << 20, 0) == B.ELORA_E_ALIGN
    assert B.lib.elora_workspace_init(FAKE, 100, 0) == B.ELORA_E_STORAGE
    assert B.lib.elora_debug_spin_limit(-1) == B.ELORA_E_SHAPE
    assert B.lib.elora_debug_spin_limit(1 << 22) == B.ELORA_OK
    assert B.lib.elora_debug_xcd_local(1) == B.ELORA_E_SHAPE
    assert B.lib.elora_debug_xcd_local(-1) == B.ELORA_OK
    assert B.lib.elora_profile_arm(-1) == B.ELORA_E_SHAPE
    assert B.lib.elora_profile_arm(0) == B.ELORA_OK


def test_workspace_grows_with_rows_and_holds_the_copy_of_a_4bit_w(B):
    # a workspace sized for more rows must hold the layout of every smaller call; from 768 rows on it also holds
    # a bf16 copy of W (d_out x d_in x 2 bytes) for the 4-bit path
    K, N, R = 1024, 768, 16
    sizes = [B.elora_workspace_bytes_w(t, K, N, R, B.ELORA_W_INT4_G32) for t in (1, 64, 65, 767, 768, 769, 4096)]
    assert all(a <= b for a, b in zip(sizes, sizes[1:]))
    assert sizes[4] - sizes[3] >= K * N * 2
    assert sizes[5] - sizes[4] < 4096
    # a W in the dtype of x needs no such copy: the workspace stays small at any row count
    same = [B.elora_workspace_bytes(t, K, N, R) for t in (1, 64, 65, 767, 768, 769, 4096)]
    assert all(a <= b for a, b in zip(same, same[1:]))
    assert same[4] - same[3] < 4096 and same[:4] == sizes[:4]
    assert same == [B.elora_workspace_bytes_w(t, K, N, R, B.ELORA_W_SAME) for t in (1, 64, 65, 767, 768, 769, 4096)]
    assert B.elora_workspace_bytes_w(64, K, N, R, 7) == 0
    # a 4-bit call with the smaller workspace is refused
    d = _desc(B, None, n_tokens=768, d_in=K, d_out=N, wfmt=B.ELORA_W_INT4_G32, w_scales=FAKE, workspace_bytes=same[4])
    assert _plan_status(B, d) == B.ELORA_E_STORAGE
    d = _desc(B, None, n_tokens=768, d_in=K, d_out=N, wfmt=B.ELORA_W_INT4_G32, w_scales=FAKE, workspace_bytes=sizes[4])
    assert _plan_status(B, d) == B.ELORA_OK
    # an 8-bit W: the copy from 257 rows on (what the decode kernel does not take), none below
    s8 = [B.elora_workspace_bytes_w(t, K, N, R, B.ELORA_W_INT8_G32) for t in (1, 64, 256, 257, 4096)]
    assert all(a <= b for a, b in zip(s8, s8[1:]))
    assert s8[3] - s8[2] >= K * N * 2 and s8[:3] == [B.elora_workspace_bytes(t, K, N, R) for t in (1, 64, 256)]
    d = _desc(B, None, n_tokens=257, d_in=K, d_out=N, wfmt=B.ELORA_W_INT8_G32, w_scales=FAKE, workspace_bytes=s8[2])
    assert _plan_status(B, d) == B.ELORA_E_STORAGE
    d = _desc(B, None, n_tokens=257, d_in=K, d_out=N, wfmt=B.ELORA_W_INT8_G32, w_scales=FAKE, workspace_bytes=s8[3])
    assert _plan_status(B, d) == B.ELORA_OK
    # group-wise formats need bf16, d_in % 32 == 0 and their scales
    assert _plan_status(B, _desc(B, None, n_tokens=4, d_in=K, d_out=N, wfmt=B.ELORA_W_INT8_G32, w_scales=None)) == B.ELORA_E_NULL
    assert _plan_status(B, _desc(B, None, n_tokens=4, d_in=48, d_out=N, wfmt=B.ELORA_W_INT8_G32, w_scales=FAKE)) == B.ELORA_E_SHAPE
    assert _plan_status(B, _desc(B, None, n_tokens=4, d_in=K, d_out=N, dtype=B.ELORA_F32, wfmt=B.ELORA_W_INT8_G32, w_scales=FAKE)) == B.ELORA_E_DTYPE
