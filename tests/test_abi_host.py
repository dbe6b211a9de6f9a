"""Host-side logic of the C ABI: the library loads, exports every declared symbol, and its
pure-host validation / workspace sizing behave as include/fq.h says.  No GPU call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fq():
    from paper_2511_12653_amd import build
    if build.stale():
        build.build()
    from paper_2511_12653_amd import binding
    return binding


def test_exports_every_declared_symbol(fq):
    hdr = open(os.path.join(ROOT, "include", "fq.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"\b(fq_[a-z_]+)\s*\(", hdr)
    assert set(names) >= {"fq_forward", "fq_backward", "fq_multi_tensor", "fq_workspace_bytes",
                          "fq_validate", "fq_status_string", "fq_workspace_init", "fq_plan_create",
                          "fq_plan_run", "fq_plan_run_adam", "fq_plan_destroy",
                          "fq_distill_loss", "fq_distill_workspace_bytes", "fq_layout"}
    lib = ctypes.CDLL(fq.library_path())
    for n in set(names):
        assert getattr(lib, n) is not None


def test_struct_size_matches_header(fq):
    # 3*8 + 3*4 + 3*4 + 4 (flags) = 52 -> padded to 56, then 9 pointers
    assert ctypes.sizeof(fq.FqTensor) == 56 + 10 * 8
    assert ctypes.sizeof(fq.FqAdam) == 4 * 8 + 8 + 3 * 8


def _desc(fq, **kw):
    base = dict(outer=2, channels=3, inner=100, dtype=fq.FQ_F16, qmin=-128, qmax=127, eps=0.0,
                s_min=fq.FLT_MIN, s_max=float("inf"), flags=0, x=0x10000, y=0x20000, q=None,
                theta=0x30000, s=None, gy=0x40000, gx=0x50000, gs=None, gtheta=0x60000)
    base.update(kw)
    return fq.FqTensor(**base)


def test_validate_ok_and_status_strings(fq):
    assert fq.fq_validate(_desc(fq), fq.FQ_MODE_FORWARD) == 0
    assert fq.fq_validate(_desc(fq), fq.FQ_MODE_BACKWARD) == 0
    assert fq.fq_status_string(0) == "ok"
    for code in range(-10, 0):
        assert fq.fq_status_string(code) not in ("ok", "unknown status")
    assert fq.fq_status_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,mode,code", [
    (dict(x=None), 1, -1), (dict(y=None), 1, -1), (dict(y=None, q=0x70000, qmax=300), 1, -4), (dict(theta=None), 1, -1),
    (dict(gy=None), 2, -1), (dict(gx=None), 2, -1),
    (dict(dtype=7), 1, -2),
    (dict(outer=-1), 1, -3), (dict(inner=1 << 62, outer=4), 1, -3), (dict(outer=1 << 31), 1, -3),
    (dict(qmin=1), 1, -4), (dict(qmin=0, qmax=0), 1, -4), (dict(qmax=40000), 1, -4),
    (dict(q=0x70000, qmin=-129), 1, -4), (dict(q=0x70000, qmax=128), 1, -4),
    (dict(x=0x10001), 1, -5), (dict(theta=0x30002), 1, -5), (dict(dtype=1, y=0x20002), 1, -5),
    (dict(gx=0x50001), 2, -5),
    (dict(s_min=0.0), 1, -7), (dict(s_min=1.0, s_max=0.5), 1, -7), (dict(eps=float("nan")), 1, -7),
    (dict(eps=float("inf")), 1, -7), (dict(s_min=float("nan")), 1, -7),
    (dict(y=0x10010), 1, -9), (dict(gx=0x40010), 2, -9),
])
def test_validate_errors(fq, kw, mode, code):
    assert fq.fq_validate(_desc(fq, **kw), mode) == code
    assert fq.fq_workspace_bytes(_desc(fq, **kw), mode) == 0


def test_validate_accepts_edge_cases(fq):
    assert fq.fq_validate(_desc(fq, y=0x10000), 1) == 0                       # exact in-place
    assert fq.fq_validate(_desc(fq, gx=0x40000), 2) == 0
    assert fq.fq_validate(_desc(fq, gx=None, flags=fq.FQ_FLAG_NO_DX), 2) == 0
    assert fq.fq_validate(_desc(fq, outer=0, x=None, y=None), 1) == 0          # empty tensor
    assert fq.fq_validate(_desc(fq, channels=0, theta=None, x=None, y=None), 1) == 0
    assert fq.fq_validate(_desc(fq, qmin=-8, qmax=7), 1) == 0
    assert fq.fq_validate(_desc(fq, y=None, q=0x70000), 1) == 0                 # codes only
    assert fq.fq_validate(_desc(fq, qmin=-127, qmax=127, q=0x70000), 1) == 0
    assert fq.fq_validate(_desc(fq, x=0x10002), 1) == 0                        # 2-byte aligned FP16
    assert fq.fq_validate([], 1) == 0
    # bad mode / list errors
    assert fq.fq_validate(_desc(fq), 3) == -3
    assert fq.fq_validate([_desc(fq), _desc(fq, dtype=9)], 1) == -2


def test_validate_adam(fq):
    def with_adam(**kw):
        a = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1, m=0x80000, v=0x90000, theta_out=0x30000)
        a.update(kw)
        return _desc(fq).set_adam(fq.FqAdam(**a))
    assert fq.fq_validate(with_adam(), 2) == 0
    assert fq.fq_validate(with_adam(), 1) == 0                       # ignored by the forward pass
    for kw in (dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(lr=float("inf")), dict(eps=-1.0)):
        assert fq.fq_validate(with_adam(**kw), 2) == -10
    assert fq.fq_validate(with_adam(m=None), 2) == -1
    assert fq.fq_validate(with_adam(v=0x90002), 2) == -5


def test_workspace_bytes(fq):
    import paper_2511_12653_amd.binding as b
    t = _desc(fq, outer=15, channels=128, inner=19200, x=1 << 32, y=2 << 32, gy=3 << 32, gx=4 << 32)                # FP16: 8 elems / vector
    # 19200 elements = 2400 vectors -> 2 chunks of 1200 per slab -> 3840 blocks, one binary64 partial each
    fwd = fq.fq_workspace_bytes(t, 1)
    bwd = fq.fq_workspace_bytes(t, 2)
    assert fwd % 256 == 0 and bwd % 256 == 0 and fwd >= 256
    # 30 blocks per channel: more than 16, so each channel has 16 first-level ticket slots beside its own
    assert bwd >= fwd + 3840 * 8 + 128 * 17 * 8
    assert bwd <= fwd + 3840 * 8 + 128 * 17 * 8 + 3 * 256
    # one scale for 7 372 800 FP16 elements = 921 600 vectors: 720 blocks of 1280 vectors share the
    # channel, more than 64, so it gets 32 first-level ticket slots beside its own: 33 slots
    pt = _desc(fq, outer=1, channels=1, inner=7372800, x=1 << 32, y=2 << 32, gy=3 << 32, gx=4 << 32)
    assert fq.fq_workspace_bytes(pt, 2) == fq.fq_workspace_bytes(pt, 1) + (720 * 8 + 128) + 512
    # 16 blocks per channel still share one slot; 18 get 16 first-level slots each
    few = _desc(fq, outer=8, channels=384, inner=19200, x=1 << 32, y=2 << 32, gy=3 << 32, gx=4 << 32)
    assert fq.fq_workspace_bytes(few, 2) == fq.fq_workspace_bytes(few, 1) + 8 * 384 * 2 * 8 + 384 * 8
    more = _desc(fq, outer=9, channels=384, inner=19200, x=1 << 32, y=2 << 32, gy=3 << 32, gx=4 << 32)
    assert fq.fq_workspace_bytes(more, 2) == fq.fq_workspace_bytes(more, 1) + 9 * 384 * 2 * 8 + 384 * 17 * 8
    # short slabs (100 FP16 elements): one wavefront per slab, one partial per slab, 2 blocks for 6 slabs
    short = _desc(fq, outer=2, channels=3, inner=100)
    assert fq.fq_workspace_bytes(short, 2) == fq.fq_workspace_bytes(short, 1) + 256 + 256
    two = fq.fq_workspace_bytes([t, t], 2)
    assert two >= 2 * (3840 * 8 + 128 * 17 * 8)
    assert fq.fq_workspace_bytes([], 2) == 256
    # launching calls refuse a missing or short workspace before touching the GPU
    with pytest.raises(b.FqError) as e:
        b.fq_backward(t, None, stream=0)
    assert e.value.status == -6
    with pytest.raises(b.FqError) as e:
        b.fq_backward(t, (0x100000, bwd - 256), stream=0)
    assert e.value.status == -6
    with pytest.raises(b.FqError) as e:
        b.fq_backward(t, (0x100010, bwd), stream=0)
    assert e.value.status == -5
    with pytest.raises(b.FqError) as e:
        b.fq_multi_tensor([t], 1, None, stream=0)
    assert e.value.status == -6
    with pytest.raises(b.FqError) as e:
        b.fq_forward(_desc(fq, x=None), stream=0)
    assert e.value.status == -1


def _distill(fq, **kw):
    base = dict(n=1, channels=384, inner=19200, dtype=fq.FQ_F16, lam=0.5, eps=1e-8, upstream=1.0,
                student=0x10000000, teacher=0x20000000, gstudent=0x30000000, out=0x40000000)
    base.update(kw)
    return fq.FqDistill(**base)


def test_distill_struct_and_workspace(fq):
    assert ctypes.sizeof(fq.FqDistill) == 3 * 8 + 4 * 4 + 4 * 8
    # 384 channels, inner a multiple of 4, aligned: the fused kernel reads the pair once and needs
    # only per-tile sums (2 doubles per tile of 64 FP16 positions: 300 tiles per image)
    assert fq.fq_distill_reads_of_pair(_distill(fq)) == 1
    got = fq.fq_distill_workspace_bytes(_distill(fq))
    assert got % 256 == 0 and 300 * 16 <= got < 300 * 16 + 256
    got = fq.fq_distill_workspace_bytes(_distill(fq, n=15))
    assert 15 * 300 * 16 <= got < 15 * 300 * 16 + 256
    assert fq.fq_distill_reads_of_pair(_distill(fq, gstudent=None)) == 1
    # more channels than a lane's registers hold (or inner not in whole quads, or pointers off the
    # quad's alignment): statistics kernel + gradient kernel, coefficients (2 doubles per position)
    # + per-tile sums (2 doubles per tile of 64 x 2 positions: 150 tiles of 128 positions)
    for kw in (dict(channels=520), dict(inner=19202), dict(student=0x10000002)):
        assert fq.fq_distill_reads_of_pair(_distill(fq, **kw)) == 2
        assert fq.fq_distill_reads_of_pair(_distill(fq, gstudent=None, **kw)) == 1
    P = 19200
    want = P * 16 + 150 * 16
    got = fq.fq_distill_workspace_bytes(_distill(fq, channels=520))
    assert got % 256 == 0 and want <= got < want + 2 * 256
    # a batch of 15 images: 15 * 75 tiles of 256 positions
    P = 15 * 19200
    want = P * 16 + 15 * 75 * 16
    got = fq.fq_distill_workspace_bytes(_distill(fq, n=15, channels=520, student=1 << 40, teacher=2 << 40,
                                                 gstudent=3 << 40))
    assert want <= got < want + 2 * 256
    assert fq.fq_distill_reads_of_pair(_distill(fq, dtype=7)) == 0 and fq.fq_distill_reads_of_pair(_distill(fq, n=0)) == 0
    # empty tensors validate and need only the minimum
    assert fq.fq_distill_workspace_bytes(_distill(fq, n=0)) == 256
    assert fq.fq_distill_workspace_bytes(_distill(fq, channels=0, student=None, teacher=None)) == 256


@pytest.mark.parametrize("kw, status", [
    (dict(dtype=7), -2), (dict(n=-1), -3), (dict(inner=2 ** 31, n=2), -3), (dict(channels=2 ** 31), -3),
    (dict(student=None), -1), (dict(teacher=None), -1), (dict(out=None), -1),
    (dict(out=0x40000004), -5), (dict(student=0x10000001), -5), (dict(gstudent=0x30000001), -5),
    (dict(eps=-1.0), -7), (dict(lam=float("nan")), -7), (dict(upstream=float("nan")), -7),
    (dict(gstudent=0x10000000 + 2), -9), (dict(gstudent=0x20000000 - 64), -9),
])
def test_distill_rejects(fq, kw, status):
    d = _distill(fq, **kw)
    assert fq.fq_distill_workspace_bytes(d) == 0
    with pytest.raises(fq.FqError) as e:
        fq.fq_distill_loss(d, (0x50000000, 1 << 40), stream=0)
    assert e.value.status == status


def test_distill_workspace_errors_before_any_launch(fq):
    d = _distill(fq)
    need = fq.fq_distill_workspace_bytes(d)
    for ws, status in [((0, need), -6), ((0x50000000, need - 1), -6), ((0x50000010, need), -5)]:
        with pytest.raises(fq.FqError) as e:
            fq.fq_distill_loss(d, ws, stream=0)
        assert e.value.status == status
    # in place over the student or the teacher is accepted
    assert fq.fq_distill_workspace_bytes(_distill(fq, gstudent=0x10000000)) == need
    assert fq.fq_distill_workspace_bytes(_distill(fq, gstudent=0x20000000)) == need


def test_codes_may_not_share_memory_with_x_or_y(fq):
    # the int8 codes are one byte per element; overlapping x (or y) in any way is refused
    for kw in (dict(q=0x1000), dict(q=0x1000 + 100), dict(q=0x2000 + 8)):
        d = _desc(fq, x=0x1000, y=0x2000, **kw)
        assert fq.fq_validate(d, fq.FQ_MODE_FORWARD) == -9
    assert fq.fq_validate(_desc(fq, x=0x1000, y=0x2000, q=0x3000), fq.FQ_MODE_FORWARD) == 0


def test_layout_info(fq):
    big = dict(x=1 << 32, y=2 << 32, gy=3 << 32, gx=4 << 32)
    # the headline tensor: 2 blocks of 1200 vectors per slab, exchange between the two
    i = fq.fq_layout(_desc(fq, outer=1, channels=384, inner=19200, **big))
    assert (i.blocks, i.units_per_channel, i.unit_elems, i.wave_units, i.extra_slots) == (768, 2, 9600, 0, 0)
    # a 188 x 120 map: four blocks per channel, the exchange tree with its two pair slots
    i = fq.fq_layout(_desc(fq, outer=1, channels=384, inner=22560, **big))
    assert (i.units_per_channel, i.wave_units, i.extra_slots) == (4, 0, 2)
    # 15 frames: 30 blocks per channel, two-level tickets with 16 first-level slots
    i = fq.fq_layout(_desc(fq, outer=15, channels=128, inner=19200, **big))
    assert (i.blocks, i.units_per_channel, i.extra_slots) == (3840, 30, 16)
    # one scale for everything: 720 blocks, 32 first-level slots
    i = fq.fq_layout(_desc(fq, outer=1, channels=1, inner=7372800, **big))
    assert (i.blocks, i.units_per_channel, i.extra_slots) == (720, 720, 32)
    # short slabs: a wavefront per slab (30 x 40 FP16 = 150 vectors), units per channel = outer
    i = fq.fq_layout(_desc(fq, outer=15, channels=384, inner=1200, **big))
    assert (i.blocks, i.units_per_channel, i.unit_elems, i.wave_units, i.extra_slots) == (1440, 15, 1200, 1, 0)
    # the same short slabs in a small tensor: a block per slab (the launch has no blocks to spare)
    i = fq.fq_layout(_desc(fq, outer=3, channels=5, inner=1000, **big))
    assert (i.blocks, i.units_per_channel, i.wave_units, i.extra_slots) == (15, 3, 0, 2)
    assert fq.fq_layout(_desc(fq, outer=1, channels=4095, inner=1000, **big)).wave_units == 0
    assert fq.fq_layout(_desc(fq, outer=1, channels=4096, inner=1000, **big)).wave_units == 1
    # 319 vectors still go to one wavefront, 320 do not (one vector is kept for a misaligned head)
    assert fq.fq_layout(_desc(fq, outer=1, channels=5000, inner=319 * 8, **big)).wave_units == 1
    assert fq.fq_layout(_desc(fq, outer=1, channels=5000, inner=320 * 8, **big)).wave_units == 0
    # in a list the switch follows the whole launch: the small tensor rides along with a large one
    small = _desc(fq, outer=3, channels=5, inner=1000, **big)
    large = _desc(fq, outer=15, channels=128, inner=19200, **big)
    alone = fq.fq_workspace_bytes([small], 2)
    both = fq.fq_workspace_bytes([small, large], 2)
    only_large = fq.fq_workspace_bytes([large], 2)
    # alone: 15 partials + 5 * 3 slots; in the list: still 15 partials (one per slab) and the same slots,
    # so the sizes add up except for the shared table
    assert alone > 256 and both <= alone + only_large
    # empty
    i = fq.fq_layout(_desc(fq, outer=0, channels=4, inner=9))
    assert (i.blocks, i.units_per_channel, i.wave_units) == (0, 0, 0)


def test_static_backward_refuses_what_its_scratch_cannot_hold(fq):
    """fq_backward_static validates and sizes on the host before it touches the GPU: descriptors
    that do not validate give their own code, tensors with more partial sums or slots than the
    built-in scratch array holds give FQ_ERR_WORKSPACE."""
    lib = ctypes.CDLL(fq.library_path())
    lib.fq_backward_static.argtypes = [ctypes.POINTER(fq.FqTensor), ctypes.c_void_p]
    lib.fq_backward_static.restype = ctypes.c_int
    call = lambda d: lib.fq_backward_static(ctypes.byref(d), None)
    assert lib.fq_backward_static(None, None) == -1
    assert call(_desc(fq, gy=None)) == -1
    assert call(_desc(fq, qmin=5)) == -4
    # one scale over 98305 chunks of 10240 FP16 elements: one partial sum too many
    big = _desc(fq, outer=1, channels=1, inner=98305 * 10240, x=1 << 40, gy=2 << 40, gx=3 << 40)
    info = fq.fq_layout(big)
    assert info.units_per_channel == 98305
    assert call(big) == -6
    # 40000 channels of one short slab each: more slots than the scratch array has
    assert call(_desc(fq, outer=1, channels=40000, inner=8, x=1 << 40, gy=2 << 40, gx=3 << 40)) == -6
    hdr = open(os.path.join(ROOT, "include", "fq.h")).read()
    assert "#define FQ_STATIC_MAX_UNITS 98304" in hdr and "#define FQ_STATIC_MAX_SLOTS 32768" in hdr
