"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol that
include/lasp2.h declares, and every argument error is reported before any device work."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_07563_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: the calls below fail earlier
ODD = ctypes.c_void_p(0x1004)


def _desc(**kw):
    base = dict(B=1, H=2, N=1024, d=64, C=128, L=0, dtype=B.LASP2_F32, n_seqs=0,
                cu_seqlens_host=None, cu_seqlens_dev=None)
    base.update(kw)
    return B.Desc(**base)


def _slots(desc):
    out = ctypes.c_int64(-1)
    rc = B.lib().lasp2_num_slots(ctypes.byref(desc), ctypes.byref(out))
    return rc, out.value


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "lasp2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(lasp2_[a-z0-9_]+)\s*\(", text))
    assert {"lasp2_chunk_states", "lasp2_state_prefix", "lasp2_attn_fwd", "lasp2_attn_bwd",
            "lasp2_num_slots", "lasp2_workspace_size", "lasp2_status_string", "lasp2_state_total",
            "lasp2_attn_bwd_noalloc",
            "lasp2_nomask_fwd", "lasp2_nomask_bwd", "lasp2_softmax_fwd", "lasp2_softmax_bwd",
            "lasp2_softmax_workspace_size", "lasp2_softmax_fwd_share", "lasp2_softmax_bwd_share",
            "lasp2_softmax_share_workspace_size"} <= names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lasp2.h but not exported"


def test_status_strings():
    for code in range(0, -9, -1):
        assert B.status_string(code) and B.status_string(code) != "unknown status"
    assert B.status_string(-99) == "unknown status"


def test_num_slots_unpacked():
    assert _slots(_desc()) == (0, 8)
    assert _slots(_desc(N=1000)) == (0, 8)                       # ragged tail
    assert _slots(_desc(N=262144, d=128, C=256, L=4096, H=16, dtype=B.LASP2_BF16)) == (0, 64)
    assert _slots(_desc(N=5, L=512)) == (0, 1)                   # slot longer than the sequence
    assert _slots(_desc(N=0)) == (0, 0)                          # empty problem


def test_num_slots_packed_matches_rule():
    cu = np.array([0, 64, 300, 301, 1024], dtype=np.int32)
    for L, C in ((128, 128), (256, 128), (512, 64)):
        want = int(sum(-(-int(n) // L) for n in np.diff(cu)))
        d = _desc(C=C, L=L, n_seqs=4, cu_seqlens_host=cu.ctypes.data, cu_seqlens_dev=0x2000)
        assert _slots(d) == (0, want)


def _walk(desc, backward=0):
    out = ctypes.c_int64(-1)
    rc = B.lib().lasp2_walk_slots(ctypes.byref(desc), backward, ctypes.byref(out))
    return rc, out.value


def test_walk_slots_choice(monkeypatch):
    """How many of the caller's slots the matrix-core attention kernels walk at a time: the host's
    choice (256 CUs assumed when no device answers).  One state per chunk still gives walks as long
    as the device can keep busy; fp32, and slots that already hold a whole sequence, stay as they are."""
    monkeypatch.delenv("LASP2_WALK_SLOTS", raising=False)
    bf = dict(d=128, C=256, dtype=B.LASP2_BF16)
    # 16 heads x 32 768 tokens, one state per chunk: walks of about 2 048 (forward) / 16 384 (backward;
    # 4 096 in packed batches) tokens, halved until the launch has two rounds of workgroups (256 forward walks at a time, 128
    # backward ones, which take two workgroups each)
    assert _walk(_desc(H=16, N=32768, **bf)) == (0, 4)
    assert _walk(_desc(H=16, N=32768, **bf), 1) == (0, 8)
    # 256 sequences of 8 192 tokens: one walk per sequence (the serial-carry order of work)
    assert _walk(_desc(B=8, H=32, N=8192, **bf)) == (0, 32)
    assert _walk(_desc(B=8, H=32, N=8192, **bf), 1) == (0, 32)
    # 300 sequences would leave most CUs idle in a second round of whole sequences
    assert _walk(_desc(B=10, H=30, N=8192, **bf)) == (0, 8)
    # 16 heads x 262 144 tokens in 4 096-token slots: long enough as they are
    assert _walk(_desc(H=16, N=262144, L=4096, **bf)) == (0, 1)
    # ... for the forward; the backward, which builds its states per walk, takes four of them
    # (16 384 tokens, two rounds of 128 walks)
    assert _walk(_desc(H=16, N=262144, L=4096, **bf), 1) == (0, 4)
    # a launch the device runs in one go stays as it is
    assert _walk(_desc(H=2, N=4096, **bf)) == (0, 1)
    # fp32 takes the plain kernels: one walk per slot
    assert _walk(_desc(H=16, N=32768)) == (0, 1)
    # a slot that holds the whole sequence
    assert _walk(_desc(H=16, N=4096, L=4096, **bf)) == (0, 1)
    # packed: never longer than the longest document needs
    cu = np.array([0, 64, 300, 301, 1024], dtype=np.int32)
    d = _desc(H=400, N=1024, d=128, C=64, dtype=B.LASP2_BF16, n_seqs=4, cu_seqlens_host=cu.ctypes.data,
              cu_seqlens_dev=0x2000)
    rc, ws = _walk(d)
    assert rc == 0 and 1 <= ws <= 16
    # the override, clamped to what the arithmetic allows
    monkeypatch.setenv("LASP2_WALK_SLOTS", "3")
    assert _walk(_desc(H=16, N=32768, **bf)) == (0, 3)
    assert _walk(_desc(H=16, N=32768)) == (0, 1)
    monkeypatch.setenv("LASP2_WALK_SLOTS", "0")
    assert _walk(_desc(H=16, N=32768, **bf)) == (0, 4)
    out = ctypes.c_int64(0)
    assert B.lib().lasp2_walk_slots(None, 0, ctypes.byref(out)) == -1
    assert B.lib().lasp2_walk_slots(ctypes.byref(_desc()), 0, None) == -1


def test_workspace_size():
    out = ctypes.c_size_t(0)
    d = _desc(B=8, H=32, N=8192, d=128, C=256, dtype=B.LASP2_BF16)
    assert B.lib().lasp2_workspace_size(ctypes.byref(d), ctypes.byref(out)) == 0
    assert out.value == 8 * 32 * 32 * 128 * 128 * 4 + 8 * 32 * 32 * 4      # states, then one counter per slot


@pytest.mark.parametrize("kw,code", [
    (dict(d=48), -2), (dict(d=256), -2), (dict(C=0), -2), (dict(C=513), -2), (dict(N=-1), -2),
    (dict(L=100), -2), (dict(L=-128), -2), (dict(B=70000, H=1), -2),
    (dict(dtype=7), -3),
    (dict(n_seqs=-1), -4),
])
def test_shape_errors(kw, code):
    assert _slots(_desc(**kw))[0] == code


def test_seqlens_errors():
    good = np.array([0, 100, 1024], dtype=np.int32)
    mk = lambda cu, **kw: _desc(n_seqs=len(cu) - 1, cu_seqlens_host=cu.ctypes.data,
                                cu_seqlens_dev=0x2000, **kw)
    assert _slots(mk(good))[0] == 0
    assert _slots(mk(good, B=2))[0] == -4                                   # packed needs B == 1
    assert _slots(mk(np.array([1, 100, 1024], dtype=np.int32)))[0] == -4    # cu[0] != 0
    assert _slots(mk(np.array([0, 100, 1000], dtype=np.int32)))[0] == -4    # cu[n] != N
    assert _slots(mk(np.array([0, 100, 100, 1024], dtype=np.int32)))[0] == -4  # empty document
    assert _slots(mk(np.array([0, 200, 100, 1024], dtype=np.int32)))[0] == -4  # not monotone
    assert _slots(_desc(n_seqs=2, cu_seqlens_host=good.ctypes.data))[0] == -4  # device copy missing
    assert _slots(_desc(cu_seqlens_dev=0x2000))[0] == -4                    # offsets without n_seqs


def test_null_and_alignment_errors_reach_no_device():
    lib, d = B.lib(), _desc()
    r = ctypes.byref(d)
    assert lib.lasp2_num_slots(None, ctypes.byref(ctypes.c_int64())) == -1
    assert lib.lasp2_num_slots(r, None) == -1
    assert lib.lasp2_chunk_states(r, None, FAKE, FAKE, None) == -1
    assert lib.lasp2_chunk_states(r, FAKE, ODD, FAKE, None) == -6
    assert lib.lasp2_state_prefix(r, FAKE, None, 0, None) == -1
    assert lib.lasp2_state_prefix(r, ODD, FAKE, 0, None) == -6
    assert lib.lasp2_attn_fwd(r, FAKE, FAKE, FAKE, None, FAKE, None) == -1
    assert lib.lasp2_attn_fwd(r, FAKE, FAKE, FAKE, FAKE, ODD, None) == -6
    args = [FAKE] * 9
    for i in range(9):
        a = list(args); a[i] = None
        assert lib.lasp2_attn_bwd(r, *a, ctypes.c_size_t(1 << 40), None) == -1
    need = ctypes.c_size_t(0)
    lib.lasp2_workspace_size(r, ctypes.byref(need))
    assert lib.lasp2_attn_bwd(r, *args, ctypes.c_size_t(need.value - 1), None) == -5
    # the entry points without masking
    assert lib.lasp2_state_total(r, FAKE, None, None) == -1
    assert lib.lasp2_state_total(r, ODD, FAKE, None) == -6
    assert lib.lasp2_nomask_fwd(r, FAKE, None, FAKE, None) == -1
    assert lib.lasp2_nomask_fwd(r, FAKE, FAKE, ODD, None) == -6
    for i in range(9):
        a = list(args); a[i] = None
        assert lib.lasp2_nomask_bwd(r, *a, ctypes.c_size_t(1 << 40), None) == -1
    assert lib.lasp2_nomask_bwd(r, *args, ctypes.c_size_t(need.value - 1), None) == -5
    # softmax attention
    for i in range(5):
        a = [FAKE] * 5; a[i] = None
        assert lib.lasp2_softmax_fwd(r, *a, 1, None) == -1
    assert lib.lasp2_softmax_fwd(r, FAKE, FAKE, ODD, FAKE, FAKE, 0, None) == -6
    sneed = ctypes.c_size_t(0)
    assert lib.lasp2_softmax_workspace_size(r, ctypes.byref(sneed)) == 0 and sneed.value == 2 * (1 * 2 * 1024 * 4)
    for i in range(10):
        a = [FAKE] * 10; a[i] = None
        assert lib.lasp2_softmax_bwd(r, *a, ctypes.c_size_t(1 << 40), 1, None) == -1
    assert lib.lasp2_softmax_bwd(r, *([FAKE] * 10), ctypes.c_size_t(sneed.value - 1), 1, None) == -5
    # one rank's share of it: the query range must lie inside the sequence (N = 1024 here)
    i64 = ctypes.c_int64
    for qb, ql in ((-1, 10), (0, -1), (1000, 25), (1025, 0)):
        assert lib.lasp2_softmax_fwd_share(r, i64(qb), i64(ql), *([FAKE] * 5), 1, None) == -2
        assert lib.lasp2_softmax_bwd_share(r, i64(qb), i64(ql), *([FAKE] * 10), ctypes.c_size_t(1 << 40), 1, None) == -2
    assert lib.lasp2_softmax_share_workspace_size(r, i64(1025), ctypes.byref(sneed)) == -2
    assert lib.lasp2_softmax_share_workspace_size(r, i64(100), ctypes.byref(sneed)) == 0 and sneed.value == 2 * (1 * 2 * 100 * 4)
    assert lib.lasp2_softmax_fwd_share(r, i64(1024), i64(0), *([None] * 5), 1, None) == 0      # no queries: nothing to do
    for i in range(5):
        a = [FAKE] * 5; a[i] = None
        assert lib.lasp2_softmax_fwd_share(r, i64(8), i64(100), *a, 1, None) == -1
    assert lib.lasp2_softmax_bwd_share(r, i64(8), i64(100), *([FAKE] * 10), ctypes.c_size_t(sneed.value - 1), 1, None) == -5


def test_null_prefix_is_accepted_only_when_every_sequence_is_one_slot():
    """Serial-carry schedule: with one slot per sequence (document) every prefix is zero and P may
    be NULL; the call then goes on to its other checks (shown here by the misaligned pointer it
    reports next, still before any device work).  With several slots a NULL P is an error."""
    lib = B.lib()
    one = ctypes.byref(_desc(N=1024, C=128, L=1024))                     # fp32: plain kernels
    many = ctypes.byref(_desc(N=1024, C=128, L=512))
    assert lib.lasp2_attn_fwd(one, FAKE, FAKE, FAKE, None, ODD, None) == -6
    assert lib.lasp2_attn_fwd(many, FAKE, FAKE, FAKE, None, ODD, None) == -1
    # backward, plain kernels: neither P nor a workspace is needed
    assert lib.lasp2_attn_bwd(one, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, ODD, None, ctypes.c_size_t(0), None) == -6
    assert lib.lasp2_attn_bwd(many, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, ODD, None, ctypes.c_size_t(0), None) == -1
    assert lib.lasp2_attn_bwd(many, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ODD, None, ctypes.c_size_t(0), None) == -1
    # backward on the matrix cores without decay: the slots' own dM_t still go through the workspace
    mf = ctypes.byref(_desc(N=1024, d=128, C=256, L=1024, dtype=B.LASP2_BF16))
    assert lib.lasp2_attn_bwd(mf, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, ctypes.c_size_t(0), None) == -1
    assert lib.lasp2_attn_bwd(mf, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, ctypes.c_size_t(16), None) == -5
    assert lib.lasp2_attn_bwd(mf, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, ODD, FAKE, ctypes.c_size_t(1 << 30), None) == -6
    # ... with decay they walk backwards from zero and need none
    lam = np.array([0.9, 1.0], dtype=np.float32)
    md = ctypes.byref(_desc(N=1024, d=128, C=256, L=1024, dtype=B.LASP2_BF16, decay_host=lam.ctypes.data,
                            decay_dev=0x3000))
    assert lib.lasp2_attn_bwd(md, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, ODD, None, ctypes.c_size_t(0), None) == -6
    # packed: one slot per document
    cu = np.array([0, 64, 300, 301, 1024], dtype=np.int32)
    pk = lambda L: ctypes.byref(_desc(C=128, L=L, n_seqs=4, cu_seqlens_host=cu.ctypes.data, cu_seqlens_dev=0x2000))
    assert lib.lasp2_attn_fwd(pk(768), FAKE, FAKE, FAKE, None, ODD, None) == -6      # longest document: 723 tokens
    assert lib.lasp2_attn_fwd(pk(640), FAKE, FAKE, FAKE, None, ODD, None) == -1      # ... now two slots


def test_noalloc_backward_argument_errors():
    """lasp2_attn_bwd_noalloc: the same checks as lasp2_attn_bwd, and a problem whose state array
    does not fit the library's fixed device array is refused, all before any device work."""
    lib = B.lib()
    r = ctypes.byref(_desc())
    args = [FAKE] * 8
    for i in range(8):
        a = list(args); a[i] = None
        assert lib.lasp2_attn_bwd_noalloc(r, *a, None) == -1
    a = list(args); a[7] = ODD
    assert lib.lasp2_attn_bwd_noalloc(r, *a, None) == -6
    assert lib.lasp2_attn_bwd_noalloc(None, *args, None) == -1
    big = _desc(B=1, H=1, N=1025 * 256, d=128, C=256, L=256, dtype=B.LASP2_BF16)      # 1025 states of 64 KiB
    need = ctypes.c_size_t(0)
    assert lib.lasp2_workspace_size(ctypes.byref(big), ctypes.byref(need)) == 0 and need.value == 1025 * 65536 + 4112      # states + 1025 counters (rounded up to 16 bytes)
    assert need.value > B.NOALLOC_SCRATCH_BYTES
    assert lib.lasp2_attn_bwd_noalloc(ctypes.byref(big), *args, None) == -5
    text = open(os.path.join(ROOT, "include", "lasp2.h")).read()
    assert re.search(r"#define\s+LASP2_NOALLOC_SCRATCH_BYTES\s+\(\(64u << 20\) \+ \(64u << 10\)\)", text) \
        and B.NOALLOC_SCRATCH_BYTES == (64 << 20) + (64 << 10)
    # empty problems need nothing
    assert lib.lasp2_attn_bwd_noalloc(ctypes.byref(_desc(N=0)), *([None] * 8), None) == 0


def test_decay_errors():
    lam = np.array([0.9, 1.0], dtype=np.float32)
    assert _slots(_desc(decay_host=lam.ctypes.data, decay_dev=0x3000))[0] == 0
    assert _slots(_desc(decay_host=lam.ctypes.data))[0] == -8            # device copy missing
    assert _slots(_desc(decay_dev=0x3000))[0] == -8                      # host copy missing
    assert _slots(_desc(decay_host=lam.ctypes.data, decay_dev=0x3002))[0] == -6
    for bad in (0.0, -0.5, 1.5, float("nan")):
        b = np.array([0.9, bad], dtype=np.float32)
        assert _slots(_desc(decay_host=b.ctypes.data, decay_dev=0x3000))[0] == -8
    # decay is defined for the masked path only
    lib = B.lib()
    r = ctypes.byref(_desc(decay_host=lam.ctypes.data, decay_dev=0x3000))
    assert lib.lasp2_state_total(r, FAKE, FAKE, None) == -8
    assert lib.lasp2_nomask_fwd(r, FAKE, FAKE, FAKE, None) == -8
    assert lib.lasp2_nomask_bwd(r, *([FAKE] * 9), ctypes.c_size_t(1 << 40), None) == -8
    assert lib.lasp2_softmax_fwd(r, *([FAKE] * 5), 1, None) == -8


def test_empty_problem_is_ok_without_pointers():
    lib = B.lib()
    for kw in (dict(N=0), dict(B=0), dict(H=0)):
        r = ctypes.byref(_desc(**kw))
        assert lib.lasp2_chunk_states(r, None, None, None, None) == 0
        assert lib.lasp2_state_prefix(r, None, None, 0, None) == 0
        assert lib.lasp2_attn_fwd(r, None, None, None, None, None, None) == 0
        assert lib.lasp2_attn_bwd(r, *([None] * 9), ctypes.c_size_t(0), None) == 0
        assert lib.lasp2_state_total(r, None, None, None) == 0
        assert lib.lasp2_nomask_fwd(r, None, None, None, None) == 0
        assert lib.lasp2_nomask_bwd(r, *([None] * 9), ctypes.c_size_t(0), None) == 0
        assert lib.lasp2_softmax_fwd(r, *([None] * 5), 0, None) == 0
        assert lib.lasp2_softmax_bwd(r, *([None] * 10), ctypes.c_size_t(0), 0, None) == 0


def test_binding_refuses_tensors_the_kernels_could_not_trust():
    """The kernels trust their pointers; the Python binding checks what torch knows about a tensor
    before handing its address over: device memory, dense layout, dtype, element count."""
    import torch
    p = B.Problem(1, 2, 128, 16, 64, 0, "f32", device="cpu")
    t = torch.zeros((1, 2, 128, 16), dtype=torch.float32)
    with pytest.raises(ValueError, match="device memory"):
        B._ptr(t)
    with pytest.raises(ValueError, match="dtype"):
        B._rows(p, t.to(torch.bfloat16), 128, "Q")
    with pytest.raises(ValueError, match="elements"):
        B._rows(p, t[:, :, :64], 128, "Q")
    with pytest.raises(ValueError, match="float32"):
        B._f32(t.to(torch.float64), 10, "LSE")
    with pytest.raises(ValueError, match="at least"):
        B._f32(t.flatten()[:5], 10, "LSE")
    B._rows(p, None, 128, "Q")      # a missing tensor is the library's to report (LASP2_ERR_NULL)
    B._rows(p, t, 128, "Q")
