"""The C-ABI library loads without a GPU, exports every declared symbol, and validates its
arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

import paper_2503_07680_amd as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hbp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hbp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = H.load_library()
    names = declared_symbols()
    assert set(names) == set(H.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert H.hbp_status_string(0) == "ok"
    assert "unsupported" in H.hbp_status_string(3)
    assert "memory" in H.hbp_status_string(7)
    assert H.hbp_status_string(99) == "unknown status"


def desc(**kw):
    base = dict(total_tokens=256, n_samples=2, n_q_heads=4, n_kv_heads=2, d_qk=128, d_v=128)
    base.update(kw)
    return H.AttnDesc(**base)


def test_tile_rows_and_workspace_queries():
    for dims in ((64, 64), (128, 128), (192, 128)):
        assert H.hbp_tile_rows(*dims, H.HBP_FWD) > 0 and H.hbp_tile_rows(*dims, H.HBP_BWD) > 0
    with pytest.raises(H.HbpError) as e:
        H.hbp_tile_rows(96, 96, H.HBP_FWD)
    assert e.value.status == 3
    d = desc()
    assert H.hbp_fwd_tile_rows(d) == H.hbp_tile_rows(128, 128, H.HBP_FWD)           # even group: one size
    mha = desc(n_q_heads=4, n_kv_heads=4)
    assert H.hbp_fwd_tile_rows(mha) == 2 * H.hbp_tile_rows(128, 128, H.HBP_FWD)     # odd group: 256 rows
    mha.fwd_tile_rows = H.hbp_fwd_tile_rows(mha)
    assert H.hbp_workspace_bytes(mha, H.HBP_FWD) >= 4                               # and the descriptor takes it
    assert H.hbp_workspace_bytes(d, H.HBP_FWD) >= 4
    need = H.hbp_workspace_bytes(d, H.HBP_BWD)
    assert need >= 256 * 4 * 4
    assert H.hbp_profile_capacity(d, H.HBP_FWD) >= 256


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=6, n_kv_heads=4), 2),       # Hq % Hkv
    (dict(d_qk=96, d_v=96), 3),                 # unsupported dims
    (dict(total_tokens=-1), 1),
    (dict(n_q_heads=0), 1),
    (dict(fwd_tile_rows=7), 1),                 # not a tile size the forward takes
    (dict(fwd_tile_rows=256), 1),               # 256-row tiles need an odd group size (here 2)
    (dict(q_stride_h=64), 2),                   # head stride smaller than the head
    (dict(k_stride_t=100), 2),                  # not a multiple of 8 elements
    (dict(q_stride_t=(1 << 22) + 8), 2),        # token stride beyond what the kernels address in 32 bits
    (dict(v_stride_t=1 << 23), 2),
    (dict(o_stride_t=1 << 40), 2),
])
def test_descriptor_validation(kw, status):
    with pytest.raises(H.HbpError) as e:
        H.hbp_workspace_bytes(desc(**kw), H.HBP_BWD)
    assert e.value.status == status


def test_largest_token_stride_is_accepted_and_the_launch_entry_points_check_it_too():
    lib = H.load_library()
    ok = desc(q_stride_t=1 << 22, k_stride_t=1 << 22, v_stride_t=1 << 22, o_stride_t=1 << 22)
    assert H.hbp_workspace_bytes(ok, H.HBP_FWD) >= 4
    bad = desc(k_stride_t=1 << 23)
    fake = 0x1000
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(bad), fake, fake, fake, fake, fake, 1, fake, fake, fake, 1 << 20,
                                   None, None) == 2
    assert lib.hbp_varlen_attn_bwd(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, fake, fake, 1, fake, 1,
                                   fake, fake, fake, fake, 1 << 30, None, None, None) == 2


def test_launch_entry_points_reject_bad_arguments_before_touching_the_device():
    lib = H.load_library()
    d = desc()
    fake = 0x1000  # never dereferenced: every call below fails validation first
    wsf = H.hbp_workspace_bytes(d, H.HBP_FWD)
    # null descriptor
    assert lib.hbp_varlen_attn_fwd(None, fake, fake, fake, fake, fake, 1, fake, fake, fake, wsf, None, None) == 1
    # missing / misaligned / small workspace
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, 1, fake, fake, None, 0, None, None) == 5
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, 1, fake, fake, 0x1010, wsf, None, None) == 5
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, 1, fake, fake, fake, 8, None, None) == 5
    assert lib.hbp_varlen_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, 1, fake, 1,
                                   fake, fake, fake, fake, 1024, None, None, None) == 5
    # null tensors, negative tile count, misaligned tensor
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), None, fake, fake, fake, fake, 1, fake, fake, fake, wsf, None, None) == 1
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, -1, fake, fake, fake, wsf, None, None) == 1
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), 0x1008, fake, fake, fake, fake, 1, fake, fake, fake, wsf, None, None) == 1
    big = H.hbp_workspace_bytes(d, H.HBP_BWD)
    assert lib.hbp_varlen_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, fake, fake, 1, fake, 1,
                                   fake, fake, fake, fake, big, None, None, None) == 1
    assert lib.hbp_varlen_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, None, 1, fake, 1,
                                   fake, fake, fake, fake, big, None, None, None) == 1
    # more (tile, head) items than the schedulers' 32-bit counters hold
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, 2 ** 30, fake, fake, fake, wsf, None, None) == 1
    # empty problems are no-ops that launch nothing
    d0 = desc(total_tokens=0, n_samples=0)
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d0), None, None, None, None, None, 0, None, None, fake, wsf, None, None) == 0
    assert lib.hbp_varlen_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, 0, fake, fake, fake, wsf, None, None) == 0


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2503_07680_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
