"""The boundary from C: tests/c_client.c (C99, -pedantic) is compiled against include/*.h, linked
with libmpa.so and run; what it prints must equal what the Python binding gets for the same calls.
Host-only calls: no GPU needed."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import paper_2503_13737_amd as mpa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_c99_client_links_and_agrees_with_the_binding(tmp_path):
    mpa.load()
    libdir = os.path.dirname(mpa.LIB_PATH)
    exe = str(tmp_path / "c_client")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_client.c"), "-L", libdir, "-lmpa", f"-Wl,-rpath,{libdir}", "-o", exe],
                   check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    got = {}
    seqs = []
    for line in r.stdout.splitlines():
        key, _, val = line.partition(" ")
        if key == "seq":
            seqs.append([int(x) for x in val.split()])
        else:
            got[key] = val

    assert int(got["create_bad"]) == mpa.MPA_ERR_UNSUPPORTED
    assert got["status_string"] == mpa.status_string(mpa.MPA_ERR_WORKSPACE)
    assert int(got["attention_null"]) == mpa.MPA_ERR_INVALID_ARG

    s = mpa.Scheduler(32, 256, 768, 0.05, 0.1, 0.75, 4096)
    s.add_request(7, 1000, 4, 1.0, 0.1, 0.0)
    s.add_request(8, 100, 2, 1.0, 0.1, 0.0)
    info = s.next_batch(0.0)
    ids, cs, ctxl, slots, table = s.batch_arrays()
    assert int(got["num_seqs"]) == info.num_seqs and int(got["num_tokens"]) == info.num_tokens
    assert int(got["token_budget"]) == info.token_budget
    assert seqs == [[int(ids[i]), int(cs[i]), int(cs[i + 1]), int(ctxl[i])] for i in range(info.num_seqs)]
    assert int(got["slot_first"]) == int(slots[0]) and int(got["slot_last"]) == int(slots[-1])

    ctx = mpa.Context(40, 128, block_size=32)
    assert int(got["workspace"]) == ctx.workspace_bytes_for_batch(cs, ctxl)
    assert int(got["workspace_bound_holds"]) == 1
    items, counts = ctx.plan_describe(cs, ctxl)
    assert int(got["plan_items"]) == items.shape[0]
    assert [int(x) for x in got["plan_counts"].split()] == [int(x) for x in np.asarray(counts)]
