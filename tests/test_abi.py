"""The C-ABI library loads on a machine without a GPU and exports every function that
include/hanayo.h declares; host-only entry points behave as documented."""

import ctypes
import os
import re

import numpy as np
import pytest

from paper_2308_15762_amd import hanayo as hn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hanayo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hanayo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 20
    lib = ctypes.CDLL(hn.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(hn.EXPORTS) == names


def test_task_record_layout():
    assert hn.TASK_DTYPE.itemsize == 12
    assert [hn.TASK_DTYPE.fields[k][1] for k in ("kind", "chunk", "rsvd", "mb", "stage")] == [0, 1, 2, 4, 8]


def test_error_strings_and_codes():
    with pytest.raises(hn.HanayoError) as ei:
        hn.hanayo_schedule(0, 1, 1, 0)
    assert ei.value.code == hn.EINVAL and "invalid argument" in str(ei.value)
    n = ctypes.c_size_t()
    buf = np.zeros(3, dtype=hn.TASK_DTYPE)
    rc = hn._lib.hanayo_schedule(2, 1, 4, 0, buf.ctypes.data, 3, ctypes.byref(n))
    assert rc == hn.EBUFSIZE and n.value == 16
    assert hn._lib.hanayo_strerror(hn.ESTATE).decode() == "task list not executable"
    for bad in [(2, 1, 4, 2), (2, 1, 4, -1), (2, 128, 1, 0), (2, 0, 4, 0)]:
        with pytest.raises(hn.HanayoError):
            hn.hanayo_schedule(*bad)


def test_sizes_and_param_layout():
    d = hn.make_desc(2, 256, 4, 1024, 128, 2, hn.PRE_LN, hn.MASK_CAUSAL, hn.BF16)
    H, F = 256, 1024
    per_block = 4 * H + 3 * H * H + 3 * H + H * H + H + H * F + F + F * H + H
    assert hn.hanayo_weight_bytes(d) == 2 * per_block * 2
    assert hn.hanayo_grad_bytes(d) == 2 * per_block * 4
    assert hn.hanayo_act_bytes(d) == 256 * 256 * 2
    off = 0
    for blk in range(2):
        for i, cnt in enumerate([H, H, H * 3 * H, 3 * H, H * H, H, H, H, H * F, F, F * H, H]):
            assert hn.hanayo_param_span(d, blk, i) == (off, cnt)
            off += cnt
    assert hn.hanayo_stash_bytes(d) % 256 == 0 and hn.hanayo_stash_bytes(d) >= 2 * 256 * (8 * H + 2 * F) * 2
    assert hn.hanayo_workspace_bytes(d) > 0
    # the workspace holds one slot of 256 partial rows [gamma sums | beta sums] per LayerNorm of the chunk (two per
    # block): they wait there until one launch adds them all to the gradients; nothing else in it depends on the
    # number of blocks
    d3 = hn.make_desc(3, 256, 4, 1024, 128, 2, hn.PRE_LN, hn.MASK_CAUSAL, hn.BF16)
    assert hn.hanayo_workspace_bytes(d3) - hn.hanayo_workspace_bytes(d) == 2 * 256 * 2 * H * 4
    for bad in [hn.make_desc(1, 250, 4, 1024, 128, 2, 0, 1, 1), hn.make_desc(1, 256, 3, 1024, 128, 2, 0, 1, 1),
                hn.make_desc(0, 256, 4, 1024, 128, 2, 0, 1, 1), hn.make_desc(1, 256, 4, 1024, 128, 2, 2, 1, 1),
                hn.make_desc(1, 8192, 64, 1024, 128, 2, 0, 1, 1)]:
        with pytest.raises(hn.HanayoError):
            hn.hanayo_weight_bytes(bad)


def test_pack_unpack_roundtrip():
    from paper_2308_15762_amd import synth
    wl = synth.WORKLOADS["tiny_gpt_fp32"]
    d = hn.desc_for(wl)
    params = synth.chunk_params(wl, 0)
    flat = hn.pack_params(d, params)
    back = hn.unpack_params(d, flat, params)
    for k in hn.PARAM_NAMES:
        assert np.array_equal(back[0][k], params[0][k])


def test_compute_calls_fail_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    d = hn.make_desc(1, 256, 4, 1024, 128, 2, hn.PRE_LN, hn.MASK_CAUSAL, hn.BF16)
    dummy = np.zeros(1024, dtype=np.uint8)
    with pytest.raises(hn.HanayoError) as ei:
        hn.hanayo_chunk_forward(d, dummy, dummy, None, dummy, dummy, dummy)
    assert ei.value.code in (hn.EHIP, hn.EUNSUPPORTED, hn.EINVAL)


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """include/hanayo.h compiled by a C compiler (-std=c99, warnings as errors), the program linked against
    libhanayo.so and run: rank 0's list of (4, 2, 8) and its stash plan, against the oracle."""
    import shutil
    import subprocess
    from oracle import schedule as OS
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "schedule_from_c")
    libdir = os.path.dirname(hn.LIB_PATH)
    subprocess.check_call([cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_c", "schedule_from_c.c"), "-o", exe,
                           "-L", libdir, "-lhanayo", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
                           "-Wl,--allow-shlib-undefined"])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    lines = out.stdout.strip().splitlines()
    tasks = OS.schedule(4, 2, 8, 0)
    peak, _, slot = OS.stash_plan(tasks, 2)
    assert lines[0] == "peak %d" % peak
    want = ["%s %d %d %d %d" % ("FB"[t.kind], t.mb, t.chunk, t.stage, s) for t, s in zip(tasks, slot)]
    assert lines[1:] == want


def test_ends_workspace_sizes():
    d = hn.make_desc(2, 1024, 16, 4096, 1024, 4, hn.PRE_LN, hn.MASK_CAUSAL, hn.BF16)
    e = hn.EndsDesc(50304, 1024, 1)
    T, H, V = 4096, 1024, 50304
    head = hn.hanayo_head_workspace_bytes(d, e)
    # the logits, two activation-sized tensors, and the fp32 partial products of the split d_hidden GEMM
    assert head >= T * V * 2 + 2 * T * H * 2 + 4 * T * H * 4 and head % 256 == 0
    assert hn.hanayo_ends_workspace_bytes(d, e) == head + T * H * 2
    for bad in (hn.EndsDesc(50300, 1024, 1), hn.EndsDesc(50304, 1000, 1), hn.EndsDesc(0, 1024, 0), hn.EndsDesc(50304, 1024, 3)):
        with pytest.raises(hn.HanayoError):
            hn.hanayo_head_workspace_bytes(d, bad)
        with pytest.raises(hn.HanayoError):
            hn.hanayo_ends_workspace_bytes(d, bad)
