"""CPU-side checks of the C-ABI boundary: the library loads, exports every
declared symbol, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2401_05391_amd as segkv
from paper_2401_05391_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "segkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(segkv_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = segkv.load_library()
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_dims_struct_matches_header():
    text = open(os.path.join(ROOT, "include", "segkv.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} segkv_dims;", text, flags=re.S).group(1)
    fields = re.findall(r"int32_t\s+(\w+);", body)
    assert fields == [f[0] for f in binding.SegkvDims._fields_]
    assert ctypes.sizeof(binding.SegkvDims) == 4 * len(fields)


def test_status_strings():
    assert segkv.status_string(0) == "ok"
    seen = {segkv.status_string(c) for c in range(-6, 1)}
    assert len(seen) == 7
    assert segkv.status_string(-99) == "unknown status"


FAKE = 0x7f0000001000  # non-null, 16-byte aligned; never dereferenced: every call below is rejected


def _decode(dims, **kw):
    lib = segkv.load_library()
    a = dict(out=FAKE, q=FAKE, pk=FAKE, pv=FAKE, rk=FAKE, rv=FAKE, parent=FAKE, kn=None, vn=None,
             slopes=None, anc=None, ws=FAKE, ws_bytes=0)
    a.update(kw)
    return lib.segkv_sdpa_decode(a["out"], a["q"], a["pk"], a["pv"], a["rk"], a["rv"], a["parent"],
                                 a["kn"], a["vn"], a["slopes"], a["anc"], a["ws"], a["ws_bytes"],
                                 0.125, ctypes.byref(dims), None)


def test_decode_rejects_bad_arguments_without_a_device():
    good = dict(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=5, Tcap=16)
    d = segkv.make_dims(**good)
    assert _decode(d, out=None) == binding.SEGKV_INVALID_ARG
    assert _decode(d, pk=None) == binding.SEGKV_INVALID_ARG
    assert _decode(d, parent=None) == binding.SEGKV_INVALID_ARG
    assert _decode(d, kn=FAKE) == binding.SEGKV_INVALID_ARG            # only one of the pair
    assert _decode(d, q=FAKE + 8) == binding.SEGKV_MISALIGNED
    assert _decode(d, rk=FAKE + 2) == binding.SEGKV_MISALIGNED
    for bad in (dict(T=0), dict(T=17), dict(Hq=7), dict(B=0), dict(Lp=-1), dict(beam=0)):
        assert _decode(segkv.make_dims(**{**good, **bad})) == binding.SEGKV_INVALID_ARG
    for bad in (dict(D=96), dict(beam=9), dict(D=512)):
        assert _decode(segkv.make_dims(**{**good, **bad})) == binding.SEGKV_UNSUPPORTED


def test_workspace_requirement_is_enforced(planner_env):
    planner_env(SEGKV_TARGET_GROUPS=1 << 20)    # force split-KV
    d = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=512, T=5, Tcap=16)
    need = segkv.workspace_bytes(d)
    assert need > 0 and need % 16 == 0
    assert _decode(d, ws=FAKE, ws_bytes=need - 1) == binding.SEGKV_WORKSPACE_TOO_SMALL
    assert _decode(d, ws=None, ws_bytes=need) == binding.SEGKV_WORKSPACE_TOO_SMALL
    assert segkv.workspace_bytes(segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=96, Lp=512, T=5,
                                                 Tcap=16)) == 0


def test_static_scratch_entry_point_rejects_oversized_dimensions_without_a_device():
    lib = segkv.load_library()
    call = lambda d_, out=FAKE: lib.segkv_sdpa_decode_static_scratch(
        out, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None, 0.125, ctypes.byref(d_), None)
    # a response of several chunks over a large batch: 7 partials of 8192 x 128 floats
    big = segkv.make_dims(B=64, beam=4, Hq=32, Hkv=32, D=128, Lp=1024, T=1300, Tcap=1312)
    assert segkv.workspace_bytes(big) > binding.STATIC_SCRATCH_BYTES
    assert call(big) == binding.SEGKV_STATIC_SCRATCH_EXCEEDED
    assert "static buffer" in segkv.status_string(binding.SEGKV_STATIC_SCRATCH_EXCEEDED)
    header = open(os.path.join(ROOT, "include", "segkv.h")).read()
    assert re.search(r"#define SEGKV_STATIC_SCRATCH_BYTES \(16u << 20\)", header)
    assert binding.STATIC_SCRATCH_BYTES == 16 << 20
    # argument checks come first, as in segkv_sdpa_decode
    ok = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=5, Tcap=16)
    assert call(ok, out=None) == binding.SEGKV_INVALID_ARG
    assert call(segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=96, Lp=64, T=5, Tcap=16)) == binding.SEGKV_UNSUPPORTED
    assert call(segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=0, Tcap=16)) == binding.SEGKV_INVALID_ARG


def test_planner_overrides_are_read_once_and_again_only_on_reload(planner_env):
    # a stray environment variable set after the first call must not change which plan ships
    d = segkv.make_dims(B=64, beam=1, Hq=8, Hkv=8, D=128, Lp=512, T=5, Tcap=16)
    before = segkv.workspace_bytes(d)
    assert before == 0                                        # 512 units: one work-group per unit
    os.environ["SEGKV_TARGET_GROUPS"] = str(1 << 20)
    try:
        assert segkv.workspace_bytes(d) == before            # not re-read
        planner_env(SEGKV_TARGET_GROUPS=1 << 20)              # sets and reloads
        assert segkv.workspace_bytes(d) > before
    finally:
        os.environ.pop("SEGKV_TARGET_GROUPS", None)


def test_hip_error_status_carries_the_runtime_text():
    text = segkv.status_string(binding.SEGKV_HIP_ERROR)
    assert text.startswith("HIP runtime rejected a kernel launch: ")
    assert len(text) > len("HIP runtime rejected a kernel launch: ")


def test_append_rejects_bad_arguments_without_a_device():
    lib = segkv.load_library()
    d = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=5, Tcap=16)
    call = lambda rk, t: lib.segkv_append_kv(rk, FAKE, FAKE, FAKE, t, ctypes.byref(d), None)
    assert call(None, 0) == binding.SEGKV_INVALID_ARG
    assert call(FAKE, -1) == binding.SEGKV_INVALID_ARG
    assert call(FAKE, 16) == binding.SEGKV_INVALID_ARG
    assert call(FAKE + 4, 3) == binding.SEGKV_MISALIGNED


def test_probe_rejects_bad_arguments_without_a_device():
    lib = segkv.load_library()
    assert lib.segkv_stream_read_probe(None, 1024, FAKE, None) == binding.SEGKV_INVALID_ARG
    assert lib.segkv_stream_read_probe(FAKE, 1000, FAKE, None) == binding.SEGKV_INVALID_ARG
    assert lib.segkv_stream_read_probe(FAKE + 4, 1024, FAKE, None) == binding.SEGKV_MISALIGNED


def test_value_stagger_hint_is_host_only_and_bounded():
    # a placement hint: a multiple of 16 below 8192, 0 for invalid dimensions
    for kw in (dict(B=32, beam=4, Hq=64, Hkv=8, D=128, Lp=2048, T=256, Tcap=256),
               dict(B=128, beam=1, Hq=32, Hkv=32, D=128, Lp=1024, T=128, Tcap=128),
               dict(B=1, beam=4, Hq=4, Hkv=4, D=64, Lp=32, T=8, Tcap=16)):
        v = segkv.value_stagger_bytes(segkv.make_dims(**kw))
        assert 0 <= v < 8192 and v % 16 == 0
    assert segkv.value_stagger_bytes(segkv.make_dims(B=0, beam=4, Hq=4, Hkv=4, D=64, Lp=32, T=8,
                                                     Tcap=16)) == 0


def test_lineage_entry_points_reject_bad_arguments_without_a_device():
    lib = segkv.load_library()
    d = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=5, Tcap=16)
    ref = ctypes.byref(d)
    # size of the list buffer: per request a 4-word header and `capacity` entries of 4 bytes
    assert lib.segkv_lineage_bytes(ref, 64) == 2 * (4 + 64) * 4
    assert lib.segkv_lineage_bytes(ref, 62) == 0            # not a multiple of 4
    assert lib.segkv_lineage_bytes(None, 64) == 0
    upd = lib.segkv_lineage_update
    assert upd(None, 64, FAKE, 1, ref, None) == binding.SEGKV_INVALID_ARG        # no list
    assert upd(FAKE, 62, FAKE, 1, ref, None) == binding.SEGKV_INVALID_ARG        # capacity % 4
    assert upd(FAKE, 64, FAKE, 16, ref, None) == binding.SEGKV_INVALID_ARG       # 17 steps x 4 beams > 64
    assert upd(FAKE, 64, FAKE, -1, ref, None) == binding.SEGKV_INVALID_ARG
    assert upd(FAKE, 64, None, 3, ref, None) == binding.SEGKV_INVALID_ARG        # parent row needed after step 0
    assert upd(FAKE + 4, 64, FAKE, 3, ref, None) == binding.SEGKV_MISALIGNED
    dec = lib.segkv_sdpa_decode_lineage
    args = lambda lin, cap: (FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, lin, cap, None, None, None, None, FAKE, 0,
                             0.125, ref, None)
    assert dec(*args(None, 64)) == binding.SEGKV_INVALID_ARG
    assert dec(*args(FAKE, 16)) == binding.SEGKV_INVALID_ARG                     # 5 steps x 4 beams > 16
    assert dec(*args(FAKE + 8, 64)) == binding.SEGKV_MISALIGNED


def test_sequence_first_prompt_entry_point_validates_like_the_batch_first_one():
    lib = segkv.load_library()
    d = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=128, Lp=64, T=5, Tcap=16)
    call = lambda d_, out=FAKE, pk=FAKE: lib.segkv_sdpa_decode_seq_first_prompt(
        out, FAKE, pk, FAKE, FAKE, FAKE, FAKE, None, None, None, None, None, FAKE, 0, 0.125,
        ctypes.byref(d_), None)
    assert call(d, out=None) == binding.SEGKV_INVALID_ARG
    assert call(d, pk=None) == binding.SEGKV_INVALID_ARG
    assert call(d, pk=FAKE + 2) == binding.SEGKV_MISALIGNED
    bad = segkv.make_dims(B=2, beam=4, Hq=8, Hkv=2, D=96, Lp=64, T=5, Tcap=16)
    assert call(bad) == binding.SEGKV_UNSUPPORTED
    wide = segkv.make_dims(B=1 << 20, beam=1, Hq=64, Hkv=64, D=128, Lp=1, T=1, Tcap=1)
    assert call(wide) == binding.SEGKV_UNSUPPORTED           # B*Hkv*D beyond the 32-bit tile offsets


def test_workspace_size_and_static_scratch_limit_agree_over_random_dimensions():
    # host logic only: the size query is deterministic, 16-byte granular, zero exactly when one
    # work-group covers a unit, and the entry point with the static buffer rejects exactly the
    # dimensions whose need exceeds its limit (checked before any device call: no GPU here)
    import random
    lib = segkv.load_library()
    rng = random.Random(20240105)
    call = lambda d_: lib.segkv_sdpa_decode_static_scratch(
        FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None, 0.125, ctypes.byref(d_), None)
    seen_zero = seen_pos = seen_big = 0
    for _ in range(400):
        D = rng.choice([64, 128, 256])
        beam = rng.choice([1, 2, 3, 4, 8])
        Hkv = rng.choice([1, 2, 4, 8, 16, 40])
        G = rng.choice([1, 1, 2, 8])
        B = rng.choice([1, 2, 7, 32, 64, 200])
        Lp = rng.choice([0, 1, 100, 1024, 5000])
        T = rng.choice([1, 2, 17, 128, 257, 900, 1500])
        d = segkv.make_dims(B=B, beam=beam, Hq=Hkv * G, Hkv=Hkv, D=D, Lp=Lp, T=T, Tcap=-(-T // 16) * 16)
        need = segkv.workspace_bytes(d)
        assert need == segkv.workspace_bytes(d) and need % 16 == 0
        if need == 0:
            seen_zero += 1
        elif need > binding.STATIC_SCRATCH_BYTES:
            seen_big += 1
            assert call(d) == binding.SEGKV_STATIC_SCRATCH_EXCEEDED
        else:
            seen_pos += 1
            # partials are fp32: (m, l) pairs and D accumulators per query and chunk, at least two chunks
            assert need >= 2 * B * beam * Hkv * G * (D + 2) * 4
    assert seen_zero and seen_pos and seen_big


@pytest.mark.gpu
def test_mfma_rate_probe_runs_and_rejects_bad_arguments():
    # the measurement helper: a short run writes finite sums and both clocks, twice the same
    import torch
    import paper_2401_05391_amd as segkv
    from paper_2401_05391_amd.binding import SegkvError
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    ops = torch.randn(16 * 256 * 8, generator=g, device=dev, dtype=torch.float32).half()
    out = torch.full((4 * 256,), float("nan"), dtype=torch.float32, device=dev)
    clocks = torch.zeros(4 * 2, dtype=torch.int64, device=dev)
    segkv.probe_mfma_rate(ops, out, clocks, 4, 10)
    torch.cuda.synchronize()
    first = out.cpu().numpy().copy()
    assert np.all(np.isfinite(first)) and np.any(first != 0)
    assert np.all(clocks.cpu().numpy() > 0)
    segkv.probe_mfma_rate(ops, out, clocks, 4, 10)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), first)
    with pytest.raises(SegkvError):
        segkv.probe_mfma_rate(ops, out, clocks, 0, 10)
    with pytest.raises(SegkvError):
        segkv.probe_mfma_rate(ops, out, clocks, 4, 0)
