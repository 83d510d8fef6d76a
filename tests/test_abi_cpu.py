"""CPU-only: the C-ABI library loads, exports every symbol the header declares,
sizes its buffers sensibly and rejects bad calls on the host before anything is
launched (no GPU is touched by these tests)."""
import ctypes
import os
import re

import pytest

from paper_2603_14360_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "m2rnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(m2rnn_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert set(names) == set(mb.EXPORTS)
    L = mb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    seen = {mb.m2rnn_status_string(c) for c in range(8)}
    assert len(seen) == 8 and "ok" in seen


def desc(**kw):
    base = dict(B=2, T=32, N=4, K=32, V=32, io=mb.M2RNN_F32)
    base.update(kw)
    return mb.make_desc(**base)


def test_sizes():
    d = desc()
    C = mb.m2rnn_default_chunk(d)
    assert 1 <= C <= mb.m2rnn_max_chunk(d)
    assert mb.m2rnn_ckpt_bytes(d) == 2 * 4 * ((32 + C - 1) // C) * 32 * 32 * 4
    assert mb.m2rnn_workspace_bytes(d, 2) >= mb.m2rnn_workspace_bytes(d, 0)
    # with the forward's checkpoints the backward needs no room for its own
    assert mb.m2rnn_workspace_bytes(d, 2) >= mb.m2rnn_workspace_bytes(d, 1) + mb.m2rnn_ckpt_bytes(d)
    big = mb.make_desc(8, 4096, 16, 64, 64, mb.M2RNN_BF16)
    assert mb.m2rnn_workspace_bytes(big, 1) < mb.m2rnn_workspace_bytes(big, 2) - mb.m2rnn_ckpt_bytes(big) + 1024
    assert mb.m2rnn_ckpt_bytes(desc(T=0)) == 0
    d7 = desc(chunk=7)
    assert mb.m2rnn_ckpt_bytes(d7) == 2 * 4 * 5 * 32 * 32 * 4
    for io in (mb.M2RNN_F32, mb.M2RNN_BF16):
        for K in (16, 32, 64, 128):
            for V in (16, 32, 64, 128):
                dd = desc(K=K, V=V, io=io)
                assert mb.m2rnn_default_chunk(dd) >= 1
                assert mb.m2rnn_workspace_bytes(dd, 1) > 0


class FakeBuf:
    """Stands in for a device buffer in host-side validation tests."""

    def __init__(self, addr, nbytes):
        self.addr, self.nbytes = addr, nbytes

    def data_ptr(self):
        return self.addr

    def numel(self):
        return self.nbytes

    def element_size(self):
        return 1


BAD = [
    (dict(K=24), 2), (dict(V=256), 2), (dict(K=0), 2), (dict(N=0), 2), (dict(Nqk=3), 2),
    (dict(B=-1), 2), (dict(T=-5), 2), (dict(io=7), 3), (dict(flags=1), 2),
    (dict(chunk=-1), 7), (dict(chunk=1 << 20), 7),
]


@pytest.mark.parametrize("kw,code", BAD)
def test_bad_descriptor_rejected(kw, code):
    d = desc(**kw)
    A = 0x1000  # a well-aligned non-null address that is never dereferenced
    ws = FakeBuf(0x100000, 1 << 40)
    rc = mb.m2rnn_fwd(d, A, A, A, A, A, None, A, None, None, ws, check=False)
    assert rc == code
    rc = mb.m2rnn_bwd(d, A, A, A, A, A, None, None, A, None, A, A, A, A, A, None, ws, check=False)
    assert rc == code
    if code != 7:
        assert mb.m2rnn_workspace_bytes(d, 1) == 0 and mb.m2rnn_ckpt_bytes(d) == 0
    assert mb.m2rnn_default_chunk(d) == 0 or code == 7


def test_null_alignment_workspace_errors():
    d = desc()
    A = 0x1000
    big = FakeBuf(0x100000, 1 << 40)
    # required pointer missing
    assert mb.m2rnn_fwd(d, None, A, A, A, A, None, A, None, None, big, check=False) == 1
    assert mb.m2rnn_fwd(d, A, A, A, A, None, None, A, None, None, big, check=False) == 1
    assert mb.m2rnn_bwd(d, A, A, A, A, A, None, None, A, None, A, A, A, A, None, None, big,
                        check=False) == 1
    # misaligned pointer
    assert mb.m2rnn_fwd(d, A + 4, A, A, A, A, None, A, None, None, big, check=False) == 4
    assert mb.m2rnn_bwd(d, A, A, A, A, A, None, None, A + 8, None, A, A, A, A, A, None, big,
                        check=False) == 4
    # workspace too small / missing
    small = FakeBuf(0x100000, 16)
    assert mb.m2rnn_fwd(d, A, A, A, A, A, None, A, None, None, small, check=False) == 5
    assert mb.m2rnn_bwd(d, A, A, A, A, A, None, None, A, None, A, A, A, A, A, None, small,
                        check=False) == 5
    assert mb.m2rnn_fwd(d, A, A, A, A, A, None, A, None, None, None, check=False) == 1
    with pytest.raises(mb.M2RNNError):
        mb.m2rnn_fwd(d, None, A, A, A, A, None, A, None, None, big)


def test_options_validation():
    """m2rnn_fwd_opt / m2rnn_bwd_opt reject incomplete or misaligned option sets on the host."""
    d = desc()
    A = 0x1000
    big = FakeBuf(0x100000, 1 << 40)
    buf = lambda addr=0x2000: FakeBuf(addr, 64)
    fwd = lambda o: mb.m2rnn_fwd_opt(d, o, A, A, A, A, A, None, A, None, None, big, check=False)
    bwd = lambda o: mb.m2rnn_bwd_opt(d, o, A, A, A, A, A, None, None, A, None, A, A, A, A, A, None,
                                     big, check=False)
    # residual weight without its gradient buffer; gate parameters without beta / gradients
    assert bwd(mb.make_opts(w_r=buf())) == 1
    assert fwd(mb.make_opts(gate=(buf(), None))) == 1
    assert bwd(mb.make_opts(gate=(buf(), buf()))) == 1
    assert bwd(mb.make_opts(gate=(buf(), buf()), dgate=(buf(), None))) == 1
    # misaligned option pointers
    assert fwd(mb.make_opts(w_r=buf(0x2004))) == 4
    assert bwd(mb.make_opts(w_r=buf(), dw_r=buf(0x2008))) == 4
    assert fwd(mb.make_opts(gate=(buf(), buf(0x2002)))) == 4
    # a bad descriptor is still reported first
    assert mb.m2rnn_fwd_opt(desc(K=24), mb.make_opts(w_r=buf()), A, A, A, A, A, None, A, None,
                            None, big, check=False) == 2


def test_static_scratch_entry_rejects_oversized_shapes_on_the_host():
    """m2rnn_fwd_static takes no workspace; a forward whose partial sums do not fit the
    library's static array is refused before any device is touched."""
    big = mb.make_desc(8, 4096, 16, 64, 64, mb.M2RNN_BF16)
    assert mb.m2rnn_workspace_bytes(big, 0) > mb.M2RNN_STATIC_SCRATCH_BYTES
    buf = FakeBuf(1 << 20, 1 << 30)
    args = [buf] * 5 + [None, buf, None, None]
    assert mb.m2rnn_fwd_static(big, None, *args, check=False) == 5
    assert mb.m2rnn_fwd_static(mb.make_desc(1, 8, 2, 24, 64, mb.M2RNN_BF16), None, *args,
                               check=False) == 2
    text = open(os.path.join(ROOT, "include", "m2rnn.h")).read()
    assert "#define M2RNN_STATIC_SCRATCH_BYTES (8u << 20)" in text


def test_every_kernel_instantiation_has_a_parity_case():
    """Host logic: every tiling and every one-wave-per-row-block shape the sources
    instantiate is reached by a case of tests/test_gpu_instantiations.py, and the dispatcher
    really routes that case's descriptor to it."""
    import importlib.util
    import sys
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    spec = importlib.util.spec_from_file_location(
        "inst_cases", os.path.join(ROOT, "tests", "test_gpu_instantiations.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    src = open(os.path.join(ROOT, "paper_2603_14360_amd", "csrc", "m2rnn_mfma_common.hpp")).read()
    src = src.replace("\\\n", " ")
    tiles = re.search(r"#define M2RNN_TILE_CASES\(X\)(.*)", src).group(1)
    rows = re.search(r"#define M2RNN_ROWWAVE_CASES\(X\)(.*)", src).group(1)
    want = {"tile<%s,%s,%s>" % t for t in re.findall(r"X\((\d+), (\d+), (\d+)\)", tiles)}
    want_rw = {"rowwave<%s,%s>" % t for t in re.findall(r"X\((\d+), (\d+)\)", rows)}
    assert len(want) >= 7 and len(want_rw) >= 12
    fwd_seen, bwd_seen = set(), set()
    for K, V, B, N, Nqk, fr, br in mod.CASES:
        d = mb.make_desc(B, 35, N, K, V, mb.M2RNN_BF16, Nqk=(Nqk or None))
        assert mb.m2rnn_route_string(d, 0) == fr and mb.m2rnn_route_string(d, 1) == br
        fwd_seen.add(fr)
        bwd_seen.add(br)
    # V = 16 tilings exist for the forward only: their backward is the register-resident one
    rwb_src = open(os.path.join(ROOT, "paper_2603_14360_amd", "csrc", "m2rnn_rowwave_bwd.hip")).read()
    rwb = re.search(r"#define M2RNN_ROWWAVE_BWD_CASES\(X\)(.*)", rwb_src).group(1)
    want_rwb = {"rowwave_bwd<%s,16>" % k for k in re.findall(r"X\((\d+)\)", rwb)}
    assert len(want_rwb) >= 2
    want_bwd = {t for t in want if not t.split(",")[1] == "16"} | want_rwb
    assert want <= fwd_seen and want_bwd <= bwd_seen, (want - fwd_seen, want_bwd - bwd_seen)
    assert want_rw <= fwd_seen, want_rw - fwd_seen


def test_block_neighbours_validate_on_the_host():
    """conv1d(4) + SiLU and gated RMSNorm entry points: sizes and refusals without a GPU."""
    buf = FakeBuf(1 << 20, 1 << 30)
    p = lambda x: ctypes.c_void_p(x.data_ptr()) if x is not None else None
    L = mb.lib()
    assert mb.m2rnn_conv_silu_workspace_bytes(2, 100, 64) > 0
    assert mb.m2rnn_conv_silu_workspace_bytes(2, 100, 12) == 0          # C not a multiple of 8
    assert mb.m2rnn_gated_rmsnorm_workspace_bytes(2, 100, 1344) > 0
    assert mb.m2rnn_gated_rmsnorm_workspace_bytes(2, 100, 8192) == 0    # D above 4096
    z = ctypes.c_void_p(0)
    assert L.m2rnn_conv_silu_fwd(2, 10, 12, 1, p(buf), p(buf), None, p(buf), z) == 2
    assert L.m2rnn_conv_silu_fwd(2, 10, 16, 5, p(buf), p(buf), None, p(buf), z) == 3
    assert L.m2rnn_conv_silu_fwd(2, 10, 16, 1, None, p(buf), None, p(buf), z) == 1
    assert L.m2rnn_conv_silu_fwd(2, 10, 16, 1, ctypes.c_void_p(buf.addr + 4), p(buf), None, p(buf), z) == 4
    assert L.m2rnn_conv_silu_bwd(2, 10, 16, 1, p(buf), p(buf), None, p(buf), p(buf), p(buf), None,
                                 p(buf), 16, z) == 5
    assert L.m2rnn_gated_rmsnorm_fwd(2, 10, 8192, 1, p(buf), p(buf), p(buf), 0.0, p(buf), None, z) == 2
    assert L.m2rnn_gated_rmsnorm_fwd(2, 10, 64, 1, p(buf), p(buf), p(buf), -1.0, p(buf), None, z) == 2
    assert L.m2rnn_gated_rmsnorm_bwd(2, 10, 64, 1, p(buf), p(buf), p(buf), 0.0, None, p(buf), p(buf),
                                     p(buf), p(buf), p(buf), 16, z) == 5
    assert L.m2rnn_gated_rmsnorm_bwd(2, 10, 64, 1, p(buf), p(buf), p(buf), 0.0, None, p(buf), None,
                                     p(buf), p(buf), p(buf), 1 << 30, z) == 1
