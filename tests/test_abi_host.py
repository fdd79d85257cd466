"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_2507_19906_amd import binding as cd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good(**kw):
    base = dict(dtype=cd.BF16, batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, window=32,
                budget=512, pool_kernel=7)
    base.update(kw)
    return cd.make_params(**base)


def test_header_symbols_are_exported():
    hdr = open(os.path.join(ROOT, "include", "calidrop.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(calidrop_[a-z_]+)\s*\(", hdr))
    assert {"calidrop_compress", "calidrop_decode", "calidrop_last_error",
            "calidrop_compress_workspace_bytes", "calidrop_decode_workspace_bytes",
            "calidrop_compress_workspace_region", "calidrop_version",
            "calidrop_recalibrate", "calidrop_recalibrate_workspace_bytes"} <= names
    L = cd.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.calidrop_version() >= 100
    assert ctypes.sizeof(cd.Params) == 56


def test_workspace_sizes():
    p = good()
    n1 = cd.calidrop_compress_workspace_bytes(p, 2 * 8192, 8192)
    n2 = cd.calidrop_compress_workspace_bytes(p, 2 * 32768, 32768)
    assert 0 < n1 < n2 and n1 % 256 == 0
    assert cd.calidrop_decode_workspace_bytes(p, 512) > 0
    off, nbytes = cd.calidrop_compress_workspace_region(p, 2 * 8192, 8192, cd.REGION_SCORE)
    assert nbytes == 2 * 8192 * 8 * 4 and off % 256 == 0 and off + nbytes <= n1
    off, nbytes = cd.calidrop_compress_workspace_region(p, 2 * 8192, 8192, cd.REGION_ROW_LSE)
    assert nbytes == 2 * 8 * 128 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=96), cd.EUNSUPPORTED),
    (dict(n_q_heads=30), cd.ESHAPE),
    (dict(n_q_heads=34, n_kv_heads=2), cd.EUNSUPPORTED),     # G = 17
    (dict(window=0), cd.EINVAL),
    (dict(budget=32), cd.EINVAL),                            # budget must exceed window
    (dict(pool_kernel=4), cd.EINVAL),
    (dict(pool_kernel=0), cd.EINVAL),
    (dict(theta1=0.9, theta2=0.5), cd.EINVAL),
    (dict(theta1=float("nan")), cd.EINVAL),
    (dict(scale=-1.0), cd.EINVAL),
    (dict(batch=0), cd.EINVAL),
    (dict(dtype=7), cd.EUNSUPPORTED),
    (dict(budget=(1 << 24) + 1), cd.EUNSUPPORTED),
])
def test_bad_params_rejected(kw, status):
    p = good(**kw)
    A = 4096     # fake, aligned, never dereferenced: validation fails first
    rc = cd.lib().calidrop_compress(ctypes.byref(p), A, A, A, A, 2 * 8192, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None)
    assert rc == status, cd.calidrop_last_error()
    assert cd.calidrop_last_error() != ""
    rc = cd.lib().calidrop_decode(ctypes.byref(p), A, A, A, A, A, 512, A, A, A, A, None, None, A,
                                  1 << 40, None)
    assert rc == status


def test_bad_struct_size_null_align_workspace():
    A = 4096
    L = cd.lib()
    p = good()
    p.struct_size = 40
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.EINVAL
    p = good()
    assert L.calidrop_compress(None, A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.EINVAL
    # null k
    assert L.calidrop_compress(ctypes.byref(p), A, None, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.EINVAL
    assert "k is NULL" in cd.calidrop_last_error()
    # misaligned v
    assert L.calidrop_compress(ctypes.byref(p), A, A, A + 8, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.EALIGN
    # workspace too small / missing / misaligned
    need = cd.calidrop_compress_workspace_bytes(p, 16384, 8192)
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A, need - 1, None) == cd.EWORKSPACE
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, None, 0, None) == cd.EWORKSPACE
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A + 16, need, None) == cd.EALIGN
    # the variant with the window rows' log-sum-exp supplied: same checks, plus its own pointer
    assert L.calidrop_compress_with_lse(ctypes.byref(p), A, A, A, A, 16384, 8192, A + 4, None, A, A, A, A, A, None, A, A, A, A, need, None) == cd.EALIGN
    assert "win_lse" in cd.calidrop_last_error()
    assert L.calidrop_compress_with_lse(ctypes.byref(p), A, None, A, A, 16384, 8192, A, None, A, A, A, A, A, None, A, A, A, A, need, None) == cd.EINVAL
    assert L.calidrop_compress_with_lse(ctypes.byref(p), A, A, A, A, 16384, 8192, A, None, A, A, A, A, A, None, A, A, A, A, need - 1, None) == cd.EWORKSPACE
    # inconsistent sizes
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 100, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.ESHAPE
    assert L.calidrop_compress(ctypes.byref(p), A, A, A, A, 3 * 8192, 8192, None, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == cd.ESHAPE      # batch*max < total
    # decode
    needd = cd.calidrop_decode_workspace_bytes(p, 512)
    assert L.calidrop_decode(ctypes.byref(p), A, A, A, A, A, 512, A, A, A, A, None, None, A,
                             needd - 1, None) == cd.EWORKSPACE
    assert L.calidrop_decode(ctypes.byref(p), A, A, A, A, A, 0, A, A, A, A, None, None, A, needd,
                             None) == cd.ESHAPE
    assert L.calidrop_decode(ctypes.byref(p), A, A, A, A, A, 512, A, A, A, None, None, None, A,
                             needd, None) == cd.EINVAL
    # cache_offsets may be NULL (uniform capacity): validation goes on to the next check ...
    assert L.calidrop_decode(ctypes.byref(p), A, A, A, None, A, 512, A, A, A, A, None, None, A,
                             needd - 1, None) == cd.EWORKSPACE
    assert L.calidrop_decode(ctypes.byref(p), A, A, A, A + 4, A, 512, A, A, A, A, None, None, A,
                             needd, None) == cd.EALIGN
    # ... unless the implied token offsets batch * max_cache_len leave the int32 range
    big = good(batch=4096)
    assert L.calidrop_decode(ctypes.byref(big), A, A, A, None, A, 1 << 20, A, A, A, A, None, None, A,
                             1 << 40, None) == cd.EUNSUPPORTED
    assert "uniform" in cd.calidrop_last_error()
    with pytest.raises(cd.CalidropError):
        cd.calidrop_compress_workspace_bytes(good(head_dim=100), 16384, 8192)
    # recalibrate
    needr = cd.calidrop_recalibrate_workspace_bytes(p, 8192)
    assert needr > 0 and needr % 256 == 0
    args = [A, A, A, A, 16384, 8192, A, None, A, A, A, A, A, A]
    assert L.calidrop_recalibrate(ctypes.byref(p), *args, A, needr - 1, None) == cd.EWORKSPACE
    args[8] = None                                          # flags is required here
    assert L.calidrop_recalibrate(ctypes.byref(p), *args, A, needr, None) == cd.EINVAL
    assert "flags is NULL" in cd.calidrop_last_error()
    args[8] = A; args[1] = A + 4
    assert L.calidrop_recalibrate(ctypes.byref(p), *args, A, needr, None) == cd.EALIGN
    assert L.calidrop_recalibrate(ctypes.byref(good(head_dim=96)), A, A, A, A, 16384, 8192, A, None, A, A, A, A, A, A,
                                  A, needr, None) == cd.EUNSUPPORTED
    # calibration size: the list of the calibration set becomes a required argument
    pc = good(calib_size=64)
    args = [A, A, A, A, 16384, 8192, A, None, A, A, A, A, A, A]
    assert L.calidrop_recalibrate(ctypes.byref(pc), *args, A, needr, None) == cd.EINVAL
    assert "cal_indices" in cd.calidrop_last_error()
    assert L.calidrop_compress(ctypes.byref(pc), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A, A,
                               1 << 40, None) == cd.EINVAL
    assert L.calidrop_compress(ctypes.byref(good(calib_size=-1)), A, A, A, A, 16384, 8192, None, A, A, A, A, A, A, A,
                               A, A, A, 1 << 40, None) == cd.EINVAL


def test_older_params_layout_is_accepted():
    # a caller compiled against the 48-byte struct (no calib_size) keeps working
    p = good()
    p.struct_size = 48
    p.calib_size = 12345            # must be ignored: it lies outside the declared size
    assert cd.calidrop_decode_workspace_bytes(p, 512) > 0
    assert cd.calidrop_compress_workspace_bytes(p, 16384, 8192) == cd.calidrop_compress_workspace_bytes(good(), 16384, 8192)
    A = 4096
    # no cal_indices needed: calib_size is 0 for this layout
    need = cd.calidrop_compress_workspace_bytes(p, 16384, 8192)
    assert cd.lib().calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A,
                                      A, need - 1, None) == cd.EWORKSPACE


def test_layout_without_flags_is_accepted_and_unknown_flags_are_rejected():
    # a caller compiled against the 52-byte struct (calib_size, no flags) keeps working: flags reads as 0
    p = good(calib_size=7)
    p.struct_size = 52
    p.flags = 0xFFFF                # must be ignored: it lies outside the declared size
    assert cd.calidrop_decode_workspace_bytes(p, 512) > 0
    A = 4096
    assert cd.lib().calidrop_compress(ctypes.byref(p), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A,
                                      A, 1 << 40, None) == cd.EINVAL
    assert "cal_indices" in cd.calidrop_last_error()       # calib_size was read, flags were not
    # per-call options: the two defined bits pass, anything else is an error before any launch
    for ok in (0, cd.OPT_WRITE_SCORES, cd.OPT_WIDE_SELECTION, cd.OPT_WRITE_SCORES | cd.OPT_WIDE_SELECTION):
        assert cd.calidrop_compress_workspace_bytes(good(flags=ok), 16384, 8192) > 0
    bad = good(flags=4)
    assert cd.lib().calidrop_compress(ctypes.byref(bad), A, A, A, A, 16384, 8192, None, A, A, A, A, A, None, A, A, A,
                                      A, 1 << 40, None) == cd.EINVAL
    assert "flags" in cd.calidrop_last_error()


def test_given_strategy_entry_points_validate_on_the_host():
    A = 4096
    L = cd.lib()
    p = good()
    need = cd.calidrop_compress_given_workspace_bytes(p, 8192)
    assert need > 0 and need % 256 == 0
    # streaming list: sink count must fit the budget
    assert L.calidrop_streaming_indices(ctypes.byref(p), -1, A, 16384, 8192, A, None) == cd.EINVAL
    assert L.calidrop_streaming_indices(ctypes.byref(p), 513, A, 16384, 8192, A, None) == cd.EINVAL
    assert "n_sink" in cd.calidrop_last_error()
    assert L.calidrop_streaming_indices(ctypes.byref(p), 32, A, 16384, 8192, None, None) == cd.EINVAL
    assert L.calidrop_streaming_indices(ctypes.byref(p), 32, A, 100, 8192, A, None) == cd.ESHAPE
    # compress_given: q_cal is required, calib_size unsupported, workspace checked
    args = [A, A, A, A, 16384, 8192, A, A, A, A, A, A, A, A]
    assert L.calidrop_compress_given(ctypes.byref(p), *args, A, need - 1, None) == cd.EWORKSPACE
    bad = list(args); bad[0] = None
    assert L.calidrop_compress_given(ctypes.byref(p), *bad, A, need, None) == cd.EINVAL
    assert "q_cal is NULL" in cd.calidrop_last_error()
    bad = list(args); bad[6] = A + 4
    assert L.calidrop_compress_given(ctypes.byref(p), *bad, A, need, None) == cd.EALIGN
    assert L.calidrop_compress_given(ctypes.byref(good(calib_size=8)), *args, A, need, None) == cd.EUNSUPPORTED
    assert L.calidrop_compress_given(ctypes.byref(good(head_dim=96)), *args, A, need, None) == cd.EUNSUPPORTED


def test_offload_entry_points_validate_on_the_host():
    A = 4096
    L = cd.lib()
    p = good()
    assert cd.calidrop_packed_rows(p, 400) == 0 and cd.calidrop_packed_rows(p, 512) == 0
    assert cd.calidrop_packed_rows(p, 8192) == 8192 - 512
    assert cd.calidrop_packed_rows(good(calib_size=100), 8192) == 100
    assert cd.calidrop_packed_rows(good(calib_size=100), 560) == 48
    with pytest.raises(cd.CalidropError):
        cd.calidrop_packed_rows(good(head_dim=100), 8192)
    needp = cd.calidrop_pack_evicted_workspace_bytes(p, 8192)
    assert needp > 0 and needp % 256 == 0
    args = [A, A, A, 16384, 8192, A, None, A, A, A, A, A]
    assert L.calidrop_pack_evicted(ctypes.byref(p), *args, A, needp - 1, None) == cd.EWORKSPACE
    bad = list(args); bad[9] = None
    assert L.calidrop_pack_evicted(ctypes.byref(p), *bad, A, needp, None) == cd.EINVAL
    assert "evict_offsets is NULL" in cd.calidrop_last_error()
    assert L.calidrop_pack_evicted(ctypes.byref(good(calib_size=8)), *args, A, needp, None) == cd.EINVAL
    assert "cal_indices" in cd.calidrop_last_error()
    needr = cd.calidrop_recalibrate_packed_workspace_bytes(p, 7680)
    assert needr > 0
    args = [A, A, A, A, A, 7680, A, A, A, A, A, A]
    assert L.calidrop_recalibrate_packed(ctypes.byref(p), *args, A, needr - 1, None) == cd.EWORKSPACE
    bad = list(args); bad[6] = None
    assert L.calidrop_recalibrate_packed(ctypes.byref(p), *bad, A, needr, None) == cd.EINVAL
    bad = list(args); bad[5] = 0
    assert L.calidrop_recalibrate_packed(ctypes.byref(p), *bad, A, needr, None) == cd.ESHAPE
    bad = list(args); bad[1] = A + 2
    assert L.calidrop_recalibrate_packed(ctypes.byref(p), *bad, A, needr, None) == cd.EALIGN


def test_h2o_entry_point_validates_on_the_host():
    A = 4096
    L = cd.lib()
    p = good()
    need = cd.calidrop_compress_h2o_workspace_bytes(p, 0, 16384, 8192)
    assert need > 0 and need % 256 == 0
    assert cd.calidrop_compress_h2o_workspace_bytes(p, 100, 16384, 8192) > 0
    for bad_local in (-1, 512, 4000):
        with pytest.raises(cd.CalidropError):
            cd.calidrop_compress_h2o_workspace_bytes(p, bad_local, 16384, 8192)
    assert "n_local" in cd.calidrop_last_error()
    args = [A, A, A, A, 16384, 8192, A, A, A, A, A, None, A, A, A]
    assert L.calidrop_compress_h2o(ctypes.byref(p), 0, *args, A, need - 1, None) == cd.EWORKSPACE
    assert L.calidrop_compress_h2o(ctypes.byref(p), 512, *args, A, need, None) == cd.EINVAL
    bad = list(args); bad[0] = None
    assert L.calidrop_compress_h2o(ctypes.byref(p), 0, *bad, A, need, None) == cd.EINVAL
    assert "q_full is NULL" in cd.calidrop_last_error()
    bad = list(args); bad[2] = A + 8
    assert L.calidrop_compress_h2o(ctypes.byref(p), 0, *bad, A, need, None) == cd.EALIGN
    assert L.calidrop_compress_h2o(ctypes.byref(good(calib_size=16)), 0, *args, A, need, None) == cd.EINVAL   # cal_indices missing
    assert L.calidrop_compress_h2o(ctypes.byref(good(batch=4096)), 0, A, A, A, A, 4096 * 8192, 8192, A, A, A, A, A, None,
                                   A, A, A, A, 1 << 44, None) == cd.EUNSUPPORTED              # batch * Hq > 65535
    off, nbytes = cd.calidrop_compress_h2o_workspace_region(p, 0, 16384, 8192, cd.REGION_VOTE_PLANES)
    assert nbytes == 16384 * 8 * 4 * 4 and off % 256 == 0 and off + nbytes <= need      # 16384*8 is a multiple of 64
    off, nbytes = cd.calidrop_compress_h2o_workspace_region(p, 0, 16384, 8192, cd.REGION_ROW_LSE)
    assert nbytes == 2 * 32 * 8192 * 4


def test_probe_library_exports_its_header():
    hdr = open(os.path.join(ROOT, "include", "calidrop_probes.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(calidrop_probe_[a-z_]+)\s*\(", hdr))
    assert names == {"calidrop_probe_stream_read", "calidrop_probe_stream_read_nt", "calidrop_probe_mfma_loop",
                     "calidrop_probe_mfma_valu", "calidrop_probe_stream_read_pieces", "calidrop_probe_stream_read_store"}
    L = ctypes.CDLL(os.path.join(ROOT, "paper_2507_19906_amd", "libcalidrop_probes.so"))
    for n in names:
        assert hasattr(L, n), n
    L.calidrop_probe_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    assert L.calidrop_probe_stream_read(None, 1 << 20, 64, 4096, None) == -1          # validation before any launch
    assert L.calidrop_probe_stream_read(4096, (1 << 20) + 16, 64, 4096, None) == -1
    L.calidrop_probe_mfma_loop.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    assert L.calidrop_probe_mfma_loop(None, 8, 8, None) == -1
    L.calidrop_probe_stream_read_pieces.argtypes = L.calidrop_probe_stream_read.argtypes
    assert L.calidrop_probe_stream_read_pieces(4096, (1 << 20) + 16, 8, 4096, None) == -1
    L.calidrop_probe_stream_read_store.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 2
    assert L.calidrop_probe_stream_read_store(4096, None, 8, 8, 5, 4096, None) == -1      # stores asked for, nowhere to put them
    L.calidrop_probe_mfma_valu.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p]
    assert L.calidrop_probe_mfma_valu(4096, 8, 8, 1, 4, 0, None) == -1             # 0 or 8 vector instructions per pair
    assert L.calidrop_probe_mfma_valu(4096, 8, 8, 0, 0, 0, None) == -1             # nothing to run


def test_append_validates_on_the_host():
    A = 4096
    L = cd.lib()
    p = good()
    assert L.calidrop_append(ctypes.byref(p), A, A, A, A, A, None, None) == cd.EINVAL
    assert "cache_lens is NULL" in cd.calidrop_last_error()
    assert L.calidrop_append(ctypes.byref(p), A + 4, A, A, A, A, A, None) == cd.EALIGN
    assert L.calidrop_append(ctypes.byref(good(head_dim=80)), A, A, A, A, A, A, None) == cd.EUNSUPPORTED


def test_public_headers_are_plain_c99(tmp_path):
    # the boundary is a C ABI: both headers must compile as C (not only as C++), pedantically
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "abi.c"
    src.write_text('#include "calidrop.h"\n#include "calidrop_probes.h"\n'
                   "int main(void) { calidrop_params p; p.struct_size = (uint32_t)sizeof(p);\n"
                   "  return (int)(sizeof(calidrop_params) != 56u) + (int)p.struct_size * 0; }\n")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                          "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
