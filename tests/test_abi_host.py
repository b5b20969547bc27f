"""CPU-only checks of the C-ABI library: it loads, exports what include/spkv.h declares,
validates configurations, and its page layout is the MFMA operand order it claims."""

import ctypes as C

import os
import re

import numpy as np
import pytest

import paper_2605_14037_amd as spkv


ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "spkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spkv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = spkv.load_library()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(spkv.EXPORTED_SYMBOLS) == names


def test_strerror_covers_all_codes():
    texts = {spkv.strerror(c) for c in range(0, -7, -1)}
    assert len(texts) == 7 and "unknown error" not in texts
    assert spkv.strerror(-99) == "unknown error"


def _cfg(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64, window=128, page_tokens=0,
                tau=0.5, max_context=4096, max_total_kept_tokens=8192)
    base.update(kw)
    return spkv.SPKVConfig(**base)


def test_required_bytes_validates_and_grows():
    base = spkv.required_bytes(_cfg())
    assert base > 0 and base % 256 == 0
    assert spkv.required_bytes(_cfg(max_total_kept_tokens=16384)) > base
    assert spkv.required_bytes(_cfg(batch=4)) > base
    for bad in (dict(batch=0), dict(batch=513), dict(n_q_heads=7), dict(head_dim=96),
                dict(window=0), dict(page_tokens=32), dict(tau=float("nan")),
                dict(max_context=0), dict(max_total_kept_tokens=-1),
                dict(n_q_heads=34, n_kv_heads=2)):
        assert spkv.required_bytes(_cfg(**bad)) == 0, bad
    # the pool term: 64 pairs * (K row + V row) per page
    more = spkv.required_bytes(_cfg(max_total_kept_tokens=8192 + 64 * 100))
    assert more - base >= 100 * 64 * 2 * 64 * 2


def test_create_rejects_bad_arguments_without_a_gpu():
    lib = spkv.load_library()
    h = C.c_void_p()
    cfg = _cfg()
    assert lib.spkv_cache_create(C.byref(cfg), None, 1 << 30, None, C.byref(h)) == -1
    assert lib.spkv_cache_create(C.byref(cfg), C.c_void_p(256), 16, None, C.byref(h)) == -1
    assert lib.spkv_cache_create(C.byref(cfg), C.c_void_p(8), 1 << 30, None, C.byref(h)) == -1
    bad = _cfg(head_dim=32)
    assert lib.spkv_cache_create(C.byref(bad), C.c_void_p(256), 1 << 30, None, C.byref(h)) == -1
    assert lib.spkv_cache_destroy(None) == -1
    assert lib.spkv_decode_attention(None, None, None, None, 0.0, None) == -1


def test_stateless_size_queries_and_null_handles():
    """The size queries that need no cache, and every entry point's refusal of a null cache
    (argument checks come before any GPU call, so they run here)."""
    lib = spkv.load_library()
    assert lib.spkv_decode_step_predict_workspace_bytes(32, 256) == 4 * 32 * 256 * 4
    assert lib.spkv_decode_step_predict_workspace_bytes(0, 256) == 0
    assert lib.spkv_decode_step_predict_workspace_bytes(32, -1) == 0
    need = lib.spkv_soft_gated_workspace_bytes(4, 8, 128, 128, 1000)
    assert need > 0 and need % 256 == 0
    assert lib.spkv_soft_gated_workspace_bytes(4, 8, 128, 128, 2000) > need
    assert lib.spkv_soft_gated_workspace_bytes(0, 8, 128, 128, 1000) == 0
    assert lib.spkv_soft_gated_workspace_bytes(4, 8, 96, 128, 1000) == 0
    assert lib.spkv_prefill_workspace_bytes(None, 16, 16) == 0
    cu = (C.c_int32 * 3)(0, 1, 2)
    assert lib.spkv_append(None, None, None, None, cu, None) == -1
    assert lib.spkv_decode_step(None, None, None, None, None, None, None, 0.0, None) == -1
    assert lib.spkv_decode_chunk(None, None, None, None, None, cu, None, None, 0.0, None) == -1
    assert lib.spkv_score_chunk(None, None, None, None, cu, None, None, 0.0, None) == -1
    assert lib.spkv_prefill_attention(None, None, None, None, None, cu, None, None, 0.0, None, 0, None) == -1
    assert lib.spkv_decode_step_predict(None, None, None, None, None, None, 128, 16, None, None, None,
                                        None, None, None, None, 0, 0.0, None) == -1
    assert lib.spkv_cache_release_sequence(None, 0, None) == -1
    assert lib.spkv_cache_set_tau(None, 0.5) == -1
    assert lib.spkv_cache_advance(None, 1) == -1


@pytest.mark.parametrize("D", [64, 128])
def test_page_layout_is_a_bijection_in_mfma_operand_order(D):
    n = 64 * D
    koff = np.array([[spkv.layout_offset(D, 0, kidx, d) for d in range(D)] for kidx in range(64)])
    voff = np.array([[spkv.layout_offset(D, 1, kidx, d) for d in range(D)] for kidx in range(64)])
    both = np.concatenate([koff.ravel(), voff.ravel()])
    assert sorted(both.tolist()) == list(range(2 * n))            # K and V tile the page exactly
    for half in range(2):
        lo = half * 2 * 32 * D
        ks = koff[half * 32:(half + 1) * 32]
        vs = voff[half * 32:(half + 1) * 32]
        assert ks.min() == lo and ks.max() == lo + 32 * D - 1     # K block, then V block
        assert vs.min() == lo + 32 * D and vs.max() == lo + 64 * D - 1
        # K tile (t, slab): lane (kc', m) holds d = 32 slab + 8 kc' + e of the tile's row m,
        # which is key 8 (m // 4) + 4 t + m % 4, at byte 16 * lane of a 1 KB tile.
        for t in range(2):
            for slab in range(D // 32):
                tile = lo + (t * (D // 8) + slab * 4) * 128
                for lane in range(64):
                    kcp, m = lane // 16, lane % 16
                    key = 8 * (m // 4) + 4 * t + m % 4
                    for e in range(8):
                        assert koff[half * 32 + key, 32 * slab + 8 * kcp + e] == tile + lane * 8 + e
        # V tile db: lane (kc, dr) holds the eight consecutive keys 8 kc + e of d = 16 db + dr,
        # and e = 4 t + i is the key that leaves row 4 kc + i of K tile t.
        for db in range(D // 16):
            tile = lo + 32 * D + db * 512
            for lane in range(64):
                kc, dr = lane // 16, lane % 16
                for e in range(8):
                    assert voff[half * 32 + 8 * kc + e, 16 * db + dr] == tile + lane * 8 + e
    assert spkv.layout_offset(D, 0, 64, 0) == -1 and spkv.layout_offset(D, 1, 0, D) == -1
    assert spkv.layout_offset(96, 0, 0, 0) == -1


def test_debug_read_rejects_bad_arguments_before_any_launch():
    lib = spkv.load_library()
    ok_ptr = C.c_void_p(4096)
    # null pointers, misaligned pointers, a run size that is no multiple of 16 KB, more runs
    # than the region holds, no workgroups
    assert lib.spkv_debug_read(None, 1 << 20, 32768, 0, 1, 1, 1, ok_ptr, None) == -1
    assert lib.spkv_debug_read(ok_ptr, 1 << 20, 32768, 0, 1, 1, 1, None, None) == -1
    assert lib.spkv_debug_read(C.c_void_p(4100), 1 << 20, 32768, 0, 1, 1, 1, ok_ptr, None) == -1
    assert lib.spkv_debug_read(ok_ptr, 1 << 20, 1000, 0, 1, 1, 1, ok_ptr, None) == -1
    assert lib.spkv_debug_read(ok_ptr, 1 << 20, 32768, 0, 33, 1, 1, ok_ptr, None) == -1
    assert lib.spkv_debug_read(ok_ptr, 1 << 20, 32768, 0, 1, 0, 1, ok_ptr, None) == -1
    assert lib.spkv_debug_read(ok_ptr, 1 << 20, 32768, 0, 1, 1, 0, ok_ptr, None) == -1


@pytest.mark.parametrize("batch,hq,hkv,D", [(512, 17, 17, 128), (512, 32, 32, 64), (512, 96, 32, 128),
                                            (300, 54, 18, 64)])
def test_arena_holds_the_multi_token_partials_of_extreme_shapes(batch, hq, hkv, D):
    """The multi-token kernels write 16, 32 or 64 columns of partial results per slot and at
    least one slot per (sequence, KV head): the arena of the largest valid shapes must have
    room for two slots of 64 columns per pair (the slot arithmetic of the host keeps one
    spare), whatever the group size."""
    pairs = batch * hkv
    need = pairs * 128 * (D + 2) * 4
    got = spkv.required_bytes(_cfg(batch=batch, n_q_heads=hq, n_kv_heads=hkv, head_dim=D,
                                   window=8, max_context=64, max_total_kept_tokens=0))
    ring = pairs * 2 * 64 * D * 2                 # one 64-pair ring page (K and V) per pair
    assert got >= need + ring
