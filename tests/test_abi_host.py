"""Host-side tests of the C ABI: the library loads without a GPU, exports what include/mpa.h
declares, rejects bad arguments before touching the GPU, and plans batches consistently."""
import ctypes
import os
import re
import time

import numpy as np
import pytest

import paper_2503_13737_amd as mpa
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(mpa_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = mpa.load()
    names = declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(mpa.EXPORTS) == names
    # the library, the header and the binding agree on the interface's version
    header = open(os.path.join(ROOT, "include", "mpa.h")).read()
    assert int(re.search(r"#define MPA_ABI_VERSION (\d+)", header).group(1)) == lib.mpa_abi_version() == mpa.MPA_ABI_VERSION


def test_create_validates_config():
    for kw, status in [(dict(num_heads=4, head_dim=96), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=4, head_dim=64, block_size=48), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=4, head_dim=64, block_size=8), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=4, head_dim=64, num_kv_heads=3), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=4, head_dim=64, num_kv_heads=8), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=4, head_dim=64, dtype=7), mpa.MPA_ERR_UNSUPPORTED),
                       (dict(num_heads=0, head_dim=64), mpa.MPA_ERR_INVALID_ARG)]:
        with pytest.raises(mpa.MpaError) as e:
            mpa.Context(**kw)
        assert e.value.status == status
    assert mpa.load().mpa_create(None, None) == mpa.MPA_ERR_INVALID_ARG
    c = mpa.Context(4, 64)
    c.close()
    mpa.Context(4, 128, dtype=mpa.MPA_FP16).close()
    assert (mpa.MPA_BF16, mpa.MPA_FP16) == (1, 2)
    assert mpa.load().mpa_destroy(None) == mpa.MPA_OK
    assert mpa.status_string(mpa.MPA_ERR_BAD_BATCH).startswith("malformed")


def test_attention_rejects_bad_arguments_without_gpu():
    lib = mpa.load()
    c = mpa.Context(4, 64)
    cs = np.array([0, 3, 4], dtype=np.int32)
    cl = np.array([5, 9], dtype=np.int32)
    fake = ctypes.c_void_p(0x1000)  # aligned, never dereferenced: every case fails validation first

    def call(q=fake, kc=fake, vc=fake, tab=fake, stride=4, cs=cs, cl=cl, S=2, T=4, out=fake, ws=fake, wsb=1 << 20):
        return lib.mpa_mixed_paged_attention(c._h, q, kc, vc, tab, stride, mpa._ptr(cs), mpa._ptr(cl), S, T,
                                             0.0, out, ws, wsb, None)

    assert call(q=None) == mpa.MPA_ERR_INVALID_ARG
    assert call(out=None) == mpa.MPA_ERR_INVALID_ARG
    assert call(q=ctypes.c_void_p(0x1004)) == mpa.MPA_ERR_INVALID_ARG
    assert call(stride=0) == mpa.MPA_ERR_INVALID_ARG
    assert call(S=-1) == mpa.MPA_ERR_INVALID_ARG
    assert call(T=5) == mpa.MPA_ERR_BAD_BATCH                       # rows do not add up
    assert call(cs=np.array([0, 3, 3], dtype=np.int32)) == mpa.MPA_ERR_BAD_BATCH   # empty sequence
    assert call(cs=np.array([1, 3, 4], dtype=np.int32)) == mpa.MPA_ERR_BAD_BATCH   # does not start at 0
    assert call(cl=np.array([2, 9], dtype=np.int32)) == mpa.MPA_ERR_BAD_BATCH      # ctx < q_len
    assert call(cl=np.array([5, 100], dtype=np.int32)) == mpa.MPA_ERR_BAD_BATCH    # table too narrow
    assert call(ws=None) == mpa.MPA_ERR_WORKSPACE
    assert call(wsb=16) == mpa.MPA_ERR_WORKSPACE
    assert call(ws=ctypes.c_void_p(0x1010)) == mpa.MPA_ERR_WORKSPACE
    # empty batch is a no-op
    assert lib.mpa_mixed_paged_attention(c._h, None, None, None, None, 0, None, None, 0, 0, 0.0, None, None, 0, None) == mpa.MPA_OK


def test_kv_append_rejects_bad_arguments_without_gpu():
    lib = mpa.load()
    c = mpa.Context(4, 64)
    fake = ctypes.c_void_p(0x1000)
    assert lib.mpa_kv_append(c._h, None, fake, fake, 3, fake, fake, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_kv_append(c._h, fake, fake, fake, -1, fake, fake, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_kv_append(c._h, fake, fake, ctypes.c_void_p(0x1004), 3, fake, fake, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_kv_append(c._h, None, None, None, 0, None, None, None) == mpa.MPA_OK
    assert lib.mpa_kv_append(None, fake, fake, fake, 3, fake, fake, None) == mpa.MPA_ERR_INVALID_ARG


def check_plan_covers(b, items, counts, H, HK=None):
    """Every (row, head, key) triple under the causal mask is covered exactly once.  Items of kind
    0 and 1 cover all heads, an item of kind 2 the query heads of K/V head kind >> 8."""
    HK = H if HK is None else HK
    G = H // HK
    ql, pr = b.q_lens, b.priors
    for i in range(b.S):
        for j in range(int(ql[i])):
            row, pos = int(b.chunk_starts[i]) + j, int(pr[i]) + j
            for kvh in range(HK):   # heads of one K/V head are always covered together
                cover = []
                for it in items:
                    seq, q_row0, q_rows, q_pos0, kb, ke, part, kind = (int(x) for x in it)
                    if (kind & 0xFF) == 2 and (kind >> 8) != kvh:
                        continue
                    if (kind & 0xFF) == 2:
                        assert G >= 4 and q_rows == 1 and 0 <= (kind >> 8) < HK
                    if q_row0 <= row < q_row0 + q_rows:
                        assert seq == i and q_pos0 + (row - q_row0) == pos
                        lo, hi = kb, min(ke, pos + 1)
                        if hi > lo:
                            cover.append((lo, hi, part))
                cover.sort()
                assert cover[0][0] == 0 and cover[-1][1] == pos + 1
                for a, bb in zip(cover, cover[1:]):
                    assert a[1] == bb[0]
                if len(cover) > 1:
                    assert all(c[2] >= 0 for c in cover)


@pytest.mark.parametrize("opts", [{}, {mpa.MPA_OPT_TG_SPLIT_BLOCKS: 1}, {mpa.MPA_OPT_PP_SPLIT_TOKENS: 64},
                                  {mpa.MPA_OPT_PP_ROWSTREAM: 1, mpa.MPA_OPT_TG_SPLIT_BLOCKS: 2}])
def test_plan_covers_every_pair_once(opts):
    b = W.config1()
    c = mpa.Context(b.H, b.D)
    for k, v in opts.items():
        c.set_option(k, v)
    items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
    assert counts[0] + counts[1] == len(items)
    assert (items[:, 4] % 16 == 0).all()
    assert (items[items[:, 7] == 1][:, 4] % 64 == 0).all()
    check_plan_covers(b, items, counts, b.H)
    need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
    assert need >= len(items) * 32
    assert c.workspace_bytes(b.S, b.T, int(b.context_lens.max())) >= need


def test_plan_large_configs_fit_upper_bound():
    for b in (W.config2(), W.config3(), W.config4()):
        c = mpa.Context(b.H, b.D)
        need = c.workspace_bytes_for_batch(b.chunk_starts, b.context_lens)
        ub = c.workspace_bytes(b.S, b.T, int(b.context_lens.max()))
        assert 0 < need <= ub, (b.name, need, ub)


def test_one_call_form_and_block_copy_reject_bad_arguments_without_gpu():
    lib = mpa.load()
    c = mpa.Context(4, 64)
    cs = np.array([0, 3, 4], dtype=np.int32)
    cl = np.array([5, 9], dtype=np.int32)
    fake = ctypes.c_void_p(0x1000)   # aligned, never dereferenced: every case fails validation first

    def call(kn=fake, vn=fake, sm=fake, q=fake, ws=fake, wsb=1 << 20, T=4):
        return lib.mpa_append_and_attend(c._h, kn, vn, sm, q, fake, fake, fake, 4, mpa._ptr(cs), mpa._ptr(cl), 2, T,
                                         0.0, fake, ws, wsb, None)

    assert call(kn=None) == mpa.MPA_ERR_INVALID_ARG
    assert call(vn=ctypes.c_void_p(0x1008)) == mpa.MPA_ERR_INVALID_ARG
    assert call(sm=ctypes.c_void_p(0x1004)) == mpa.MPA_ERR_INVALID_ARG
    assert call(q=None) == mpa.MPA_ERR_INVALID_ARG
    assert call(T=7) == mpa.MPA_ERR_BAD_BATCH
    assert call(ws=None) == mpa.MPA_ERR_WORKSPACE          # nothing is appended when the call is refused
    assert lib.mpa_append_and_attend(c._h, None, None, None, None, None, None, None, 0, None, None, 0, 0, 0.0,
                                     None, None, 0, None) == mpa.MPA_OK
    assert lib.mpa_copy_blocks(c._h, None, fake, fake, fake, fake, 3, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_copy_blocks(c._h, fake, fake, fake, fake, ctypes.c_void_p(0x1004), 3, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_copy_blocks(c._h, fake, fake, fake, fake, fake, -1, None) == mpa.MPA_ERR_INVALID_ARG
    assert lib.mpa_copy_blocks(None, fake, fake, fake, fake, fake, 1, None) == mpa.MPA_ERR_INVALID_ARG
    with pytest.raises(mpa.MpaError):
        c.set_option(mpa.MPA_OPT_PROFILE_EVERY, 0)


def test_an_upload_that_never_reports_back_fails_the_call_before_anything_is_touched():
    """The staging ring's error path, driven from the host: the buffer the next call would use is
    marked as still being read by an upload whose ticket never arrives.  The call must wait the
    configured time, then return MPA_ERR_HIP with hipErrorNotReady -- before it writes to the buffer
    or launches anything (no HIP call at all has been made when it returns: this runs without a
    GPU) -- and the next call must find the same buffer and fail the same way."""
    HIP_ERROR_NOT_READY = 600
    lib = mpa.load()
    c = mpa.Context(4, 64)
    c.set_option(mpa.MPA_OPT_STAGING_TIMEOUT_MS, 60)
    c.set_option(mpa.MPA_OPT_TEST_STUCK_UPLOAD, 1)
    with pytest.raises(mpa.MpaError):
        c.set_option(mpa.MPA_OPT_TEST_STUCK_UPLOAD, 1)        # the slot is taken already
    cs = np.array([0, 3, 4], dtype=np.int32)
    cl = np.array([5, 9], dtype=np.int32)
    fake = ctypes.c_void_p(0x1000)   # aligned, never dereferenced: the call fails before any launch
    for attempt in range(2):
        t0 = time.perf_counter()
        rc = lib.mpa_mixed_paged_attention(c._h, fake, fake, fake, fake, 4, mpa._ptr(cs), mpa._ptr(cl), 2, 4, 0.0,
                                           fake, fake, 1 << 20, None)
        dt = time.perf_counter() - t0
        assert rc == mpa.MPA_ERR_HIP and lib.mpa_last_hip_error(c._h) == HIP_ERROR_NOT_READY, attempt
        assert 0.05 <= dt < 2.0
    rc = lib.mpa_append_and_attend(c._h, fake, fake, fake, fake, fake, fake, fake, 4, mpa._ptr(cs), mpa._ptr(cl), 2, 4,
                                   0.0, fake, fake, 1 << 20, None)
    assert rc == mpa.MPA_ERR_HIP and lib.mpa_last_hip_error(c._h) == HIP_ERROR_NOT_READY
    c.close()   # a planted slot is ordinary memory and is freed


def test_options_and_measurement_aid_reject_bad_arguments_without_gpu():
    lib = mpa.load()
    c = mpa.Context(4, 64)
    for opt, bad in ((mpa.MPA_OPT_TILE_MODE, 3), (mpa.MPA_OPT_PROFILE_REPEAT, 0), (mpa.MPA_OPT_PROFILE_REPEAT, 5000),
                     (mpa.MPA_OPT_STAGING_TIMEOUT_MS, 0), (mpa.MPA_OPT_PLAN_CACHE, 3), (99, 1)):
        with pytest.raises(mpa.MpaError):
            c.set_option(opt, bad)
    for opt, good in ((mpa.MPA_OPT_TILE_MODE, 2), (mpa.MPA_OPT_TILE_MODE, 0), (mpa.MPA_OPT_PROFILE_REPEAT, 8),
                      (mpa.MPA_OPT_STAGING_TIMEOUT_MS, 100)):
        c.set_option(opt, good)
    # the work-group shape changes the tiles of the plan, not the coverage
    b = W.config1()
    c.set_option(mpa.MPA_OPT_TILE_MODE, 2)
    items, counts = c.plan_describe(b.chunk_starts, b.context_lens)
    check_plan_covers(b, items, counts, b.H)
    fake = ctypes.c_void_p(0x1000)
    call = lib.mpa_ceiling_launch
    assert call(mpa.MPA_CEIL_STREAM_READ, fake, 1 << 30, 0, None, None) == mpa.MPA_ERR_INVALID_ARG      # no sink
    assert call(mpa.MPA_CEIL_STREAM_READ, None, 1 << 30, 0, fake, None) == mpa.MPA_ERR_INVALID_ARG      # no buffer
    assert call(mpa.MPA_CEIL_STREAM_READ, fake, 1000, 0, fake, None) == mpa.MPA_ERR_INVALID_ARG         # too small
    assert call(mpa.MPA_CEIL_RANDOM_4K, fake, 1 << 30, 3, fake, None) == mpa.MPA_ERR_INVALID_ARG        # odd chunk count
    assert call(mpa.MPA_CEIL_RANDOM_16K, fake, 1 << 16, 4, fake, None) == mpa.MPA_ERR_INVALID_ARG       # fewer than 64 chunks
    assert call(mpa.MPA_CEIL_MFMA_BF16, None, 0, 0, fake, None) == mpa.MPA_ERR_INVALID_ARG              # no iterations
    assert call(mpa.MPA_CEIL_MFMA_BF16_NOISY, None, 0, 0, fake, None) == mpa.MPA_ERR_INVALID_ARG        # no iterations
    assert call(mpa.MPA_CEIL_MFMA_BF16_NOISY + 1, None, 0, 4, fake, None) == mpa.MPA_ERR_INVALID_ARG    # no such kind
    assert call(17, fake, 1 << 30, 2, fake, None) == mpa.MPA_ERR_INVALID_ARG


def test_no_exception_crosses_the_boundary_when_the_host_runs_out_of_memory():
    """In a child process whose address space is capped just above what it already uses, planning a batch
    of eight million sequences cannot allocate its work list: the call reports MPA_ERR_NO_MEMORY (no abort,
    no C++ exception through the C frames) and the context keeps working."""
    import subprocess
    import sys
    code = r'''
import resource, numpy as np
import paper_2503_13737_amd as mpa
mpa.load()
ctx = mpa.Context(4, 128)
S = 8_000_000
cs = np.arange(S + 1, dtype=np.int32)
cl = np.full(S, 40, dtype=np.int32)
small = ctx.plan_describe(cs[:3], cl[:2])[0].shape[0]
vm = int(next(l for l in open("/proc/self/status") if l.startswith("VmSize")).split()[1]) * 1024
resource.setrlimit(resource.RLIMIT_AS, (vm + (160 << 20), vm + (160 << 20)))
try:
    ctx.plan_describe(cs, cl)
    print("status", 0)
except mpa.MpaError as e:
    print("status", e.status)
print("bytes", ctx.workspace_bytes_for_batch(cs, cl))
print("again", ctx.plan_describe(cs[:3], cl[:2])[0].shape[0] == small)
'''
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300,
                       cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    assert r.returncode == 0, r.stderr[-2000:]
    got = dict(line.split() for line in r.stdout.splitlines() if line.strip())
    assert int(got["status"]) == mpa.MPA_ERR_NO_MEMORY
    assert int(got["bytes"]) == 0          # the size query reports "no valid answer" the way it does for a bad batch
    assert got["again"] == "True"
    assert mpa.status_string(mpa.MPA_ERR_NO_MEMORY) == "out of host memory"
