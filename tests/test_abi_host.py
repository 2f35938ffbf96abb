"""Host-only checks of the C ABI: the library loads, exports every function the header declares,
and rejects host-checkable argument errors before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2604_19877_amd import binding as sa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "samixers.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b([a-z_0-9]+)\s*\([^;{}]*\)\s*;", text)


def test_library_exports_every_declared_function():
    names = header_functions()
    assert len(names) >= 15 and "placement_decode" in names and "gdn_decode_step" in names
    import torch  # noqa: F401  (its HIP runtime must be loaded first, as the binding does)
    handle = ctypes.CDLL(sa.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), "libsamixers.so does not export %s" % n
    assert set(names) == set(sa.EXPORTS), "binding and header disagree"


def test_version_and_error_string():
    assert sa.sa_version() >= 100
    assert isinstance(sa.sa_last_error(), str)


def _recurrent_call(fn, **over):
    a = dict(q=16, k=16, v=16, alpha=16, beta=16, state_in=16, state_out=16, out=16, slot_idx=None, req_idx=None,
             n_req=0, B=2, T=1, H=4, Hk=4, dk=128, dv=128, scale=1.0, n_commit=1, stream=0)
    a.update(over)
    fn(**a)


@pytest.mark.parametrize("fn", [sa.gdn_decode_step, sa.kda_decode_step])
def test_recurrent_argument_errors(fn):
    with pytest.raises(sa.SaError) as e:
        _recurrent_call(fn, dk=96, dv=96)
    assert e.value.status == sa.SA_EUNSUPPORTED and "96" in str(e.value)
    for bad in (dict(T=0), dict(T=17), dict(Hk=3), dict(n_commit=2), dict(n_commit=-1), dict(q=None), dict(state_out=8),
                dict(req_idx=16, n_req=3)):
        with pytest.raises(sa.SaError) as e:
            _recurrent_call(fn, **bad)
        assert e.value.status == sa.SA_EINVAL, bad
    _recurrent_call(fn, B=0)                       # empty batch: nothing to do, no error
    _recurrent_call(fn, req_idx=16, n_req=0)       # empty request list


@pytest.mark.parametrize("fn", [sa.gdn_chunk_steps, sa.kda_chunk_steps])
def test_chunked_recurrent_argument_errors(fn):
    def call(**over):
        a = dict(q=16, k=16, v=16, alpha=16, beta=16, state_in=16, state_out=16, out=16, slot_idx=None, req_idx=None,
                 n_req=0, B=2, T=40, H=4, Hk=4, dk=128, dv=128, scale=1.0, stream=0)
        a.update(over)
        fn(**a)
    with pytest.raises(sa.SaError) as e:
        call(dk=64, dv=64)                # the one-token kernels take this shape, the chunked ones do not
    assert e.value.status == sa.SA_EUNSUPPORTED and "64" in str(e.value)
    for bad in (dict(T=0), dict(Hk=3), dict(v=None), dict(out=4), dict(req_idx=16, n_req=3), dict(B=-1)):
        with pytest.raises(sa.SaError) as e:
            call(**bad)
        assert e.value.status == sa.SA_EINVAL, bad
    call(B=0)
    call(req_idx=16, n_req=0)


def _attn_call(**over):
    a = dict(q=16, kpool=16, vpool=16, n_pages=4, page_table=16, max_pages=4, seq_lens=16, req_idx=None, n_req=0, out=16,
             B=2, T=1, Hq=32, Hkv=8, D=128, page_size=16, max_seq_len=64, window=0, scale=1.0, workspace=16,
             workspace_bytes=1 << 30, stream=0)
    a.update(over)
    sa.attn_decode(**a)


def test_attention_argument_errors():
    for bad, code in ((dict(D=64), sa.SA_EUNSUPPORTED), (dict(page_size=32), sa.SA_EUNSUPPORTED),
                      (dict(T=9), sa.SA_EUNSUPPORTED), (dict(Hq=30), sa.SA_EINVAL), (dict(max_seq_len=65), sa.SA_EINVAL),
                      (dict(workspace_bytes=16, max_pages=2048, max_seq_len=32768), sa.SA_EWORKSPACE),
                      (dict(workspace=None, max_pages=2048, max_seq_len=32768), sa.SA_EINVAL), (dict(kpool=None), sa.SA_EINVAL),
                      (dict(out=4), sa.SA_EINVAL), (dict(n_pages=0), sa.SA_EINVAL)):
        with pytest.raises(sa.SaError) as e:
            _attn_call(**bad)
        assert e.value.status == code, bad
    _attn_call(B=0)


def test_workspace_size_formula():
    # partials are (D + 2) floats per (request, query row, page range): more ranges for longer contexts
    small = sa.attn_decode_workspace_bytes(64, 1, 32, 8, 128, 4096, 0)
    big = sa.attn_decode_workspace_bytes(64, 1, 32, 8, 128, 32768, 0)
    assert small > 0 and big >= small and big % (64 * 32 * 130 * 4) == 0
    assert sa.attn_decode_workspace_bytes(64, 1, 32, 8, 128, 32768, 4096) == 0       # one range per (request, KV head)
    assert sa.attn_decode_workspace_bytes(64, 1, 32, 8, 64, 32768, 0) == 0
    # ranges per (request, KV head): at least 16 pages each, 4 or more for full attention when the context allows
    per_range = lambda n_req, ctx: sa.attn_decode_workspace_bytes(n_req, 1, 32, 8, 128, ctx, 0) // (n_req * 32 * 130 * 4)
    assert per_range(3, 2048) == 8 and per_range(64, 2048) == 4 and per_range(64, 32768) == 4

def test_kv_append_argument_errors():
    base = dict(k_new=16, v_new=16, kpool=16, vpool=16, n_pages=4, page_table=16, max_pages=4, positions=16, B=1, T=1,
                Hkv=8, D=128, page_size=16, stream=0)
    for bad, code in ((dict(D=256), sa.SA_EUNSUPPORTED), (dict(T=0), sa.SA_EINVAL), (dict(vpool=None), sa.SA_EINVAL)):
        with pytest.raises(sa.SaError) as e:
            sa.kv_append(**{**base, **bad})
        assert e.value.status == code
    sa.kv_append(**{**base, "B": 0})


def test_placement_plan_errors():
    for placements, ids in ((["FSK", "FSKG"], [0]), (["FSKX"], [0]), (["FSKG"], [1]), (["FSKG"], [-1])):
        with pytest.raises(sa.SaError) as e:
            sa.placement_plan_create(placements, ids)
        assert e.value.status == sa.SA_EINVAL


def test_state_tile_helpers_check_their_arguments():
    assert sa.sa_state_tile_bytes(128, 128) == 65536 and sa.sa_state_tile_bytes(64, 64) == 16384
    assert sa.sa_state_tile_bytes(96, 96) == 0
    for fn in (sa.sa_state_pack, sa.sa_state_unpack):
        fn(16, 1 << 20, 0, 128, 128, 0)                            # nothing to convert (stream 0: no GPU is touched)
        for bad, status in (((16, 1 << 20, 1, 96, 96), sa.SA_EUNSUPPORTED), ((None, 1 << 20, 1, 128, 128), sa.SA_EINVAL),
                            ((16, 1 << 20, -1, 128, 128), sa.SA_EINVAL), ((8, 1 << 20, 1, 128, 128), sa.SA_EINVAL),
                            ((1 << 20, (1 << 20) + 65536, 2, 128, 128), sa.SA_EINVAL)):   # the last one overlaps
            with pytest.raises(sa.SaError) as e:
                fn(*bad, 0)
            assert e.value.status == status, bad


def test_stream_tiles_checks_its_arguments():
    for bad in (dict(kind=3), dict(kind=-1), dict(n_tiles=-1), dict(tiles=None), dict(tiles=8)):
        a = dict(kind=0, tiles=16, n_tiles=4, stream=0)
        a.update(bad)
        with pytest.raises(sa.SaError) as e:
            sa.sa_stream_tiles(**a)
        assert e.value.status == sa.SA_EINVAL, bad
    sa.sa_stream_tiles(2, 16, 0, 0)   # no tiles: nothing to do, no error


@pytest.mark.parametrize("fn", [sa.gdn_decode_step_var, sa.kda_decode_step_var])
def test_per_request_commit_argument_errors(fn):
    def call(**over):
        a = dict(q=16, k=16, v=16, alpha=16, beta=16, state_in=16, state_out=16, out=16, slot_idx=None, req_idx=None,
                 n_req=0, B=2, T=4, H=4, Hk=4, dk=128, dv=128, scale=1.0, n_commit_rows=16, stream=0)
        a.update(over)
        fn(**a)
    for bad in (dict(n_commit_rows=None), dict(n_commit_rows=6), dict(T=0), dict(T=17), dict(Hk=3), dict(q=None)):
        with pytest.raises(sa.SaError) as e:
            call(**bad)
        assert e.value.status == sa.SA_EINVAL, bad
    with pytest.raises(sa.SaError) as e:
        call(dk=96, dv=96)
    assert e.value.status == sa.SA_EUNSUPPORTED
    call(B=0, n_commit_rows=None)          # empty batch: nothing to do, no error
    call(req_idx=16, n_req=0)              # empty request list
