"""CPU-side checks of the C ABI: the library loads, exports every declared
entry point, and rejects bad arguments on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2603_06938_amd import binding as sw

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "swimba.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swimba_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sw._load()
    names = declared_symbols()
    assert {"swimba_mixer_fwd", "swimba_step", "swimba_router_topk"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def dims(**kw):
    base = dict(batch=1, seqlen=256, nheads=4, headdim=16, dstate=16, ngroups=1, nexperts=4, top_k=2,
                chunk=64, io_dtype=0)
    base.update(kw)
    return sw.make_dims(**base)


def test_workspace_query_and_layout():
    d = dims()
    n = sw.swimba_mixer_workspace_bytes(d)
    lo = sw.swimba_mixer_workspace_layout(d)
    assert n == lo.total and n > 0
    offs = [lo.topk_idx, lo.topk_w, lo.cs, lo.states, lo.states_lp, lo.cmix, lo.bmix_t8, lo.bmix_frag, lo.cb]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lo.topk_w - lo.topk_idx >= 256 * 2 * 4
    assert lo.states - lo.cs >= 4 * 4 * 64 * 4
    assert lo.states_lp - lo.states >= 4 * 4 * 16 * 16 * 4
    # ragged L: one more chunk
    assert sw.swimba_mixer_workspace_bytes(dims(seqlen=257)) > n
    # the bf16 MFMA shape carries a low-precision copy of the states
    m = dims(headdim=64, dstate=128, chunk=256, io_dtype=1, seqlen=512)
    lm = sw.swimba_mixer_workspace_layout(m)
    assert lm.states_lp == lm.states          # no fp32 states on the MFMA path
    assert lm.cmix - lm.states_lp >= 2 * 4 * 64 * 128 * 2
    assert lm.bmix_t8 - lm.cmix >= 512 * 128 * 2 and lm.bmix_frag - lm.bmix_t8 >= 512 * 128 * 2
    assert lm.cb - lm.bmix_frag >= 512 * 128 * 2
    assert lm.total - lm.cb >= 2 * 36 * 2048


@pytest.mark.parametrize("kw,status", [
    (dict(io_dtype=7), 3),
    (dict(nheads=0), 2), (dict(top_k=0), 2), (dict(top_k=5), 2), (dict(ngroups=3), 2),
    (dict(chunk=0), 2), (dict(batch=-1), 2),
    (dict(chunk=512), 4), (dict(nexperts=300, top_k=2), 4), (dict(nexperts=32, top_k=17), 4),
    (dict(headdim=128, dstate=128), 4), (dict(dstate=512), 4),
])
def test_invalid_dims_are_rejected_on_the_host(kw, status):
    d = dims(**kw)
    assert sw.swimba_mixer_workspace_bytes(d) == 0
    lo = sw.swimba_ws_layout()
    assert sw._load().swimba_mixer_workspace_layout(ctypes.byref(d), ctypes.byref(lo)) == status
    # mixer_fwd reports the same status before looking at any pointer
    st = sw._load().swimba_mixer_fwd(ctypes.byref(d), *([None] * 12), None, 0, None)
    assert st == status


def test_null_and_workspace_errors_enqueue_nothing():
    lib = sw._load()
    d = dims()
    assert lib.swimba_mixer_fwd(None, *([None] * 12), None, 0, None) == 1
    # valid dims, no workspace
    assert lib.swimba_mixer_fwd(ctypes.byref(d), *([None] * 12), None, 0, None) == 5
    # misaligned / too small workspace (host-side pointer value only; never dereferenced)
    assert lib.swimba_mixer_fwd(ctypes.byref(d), *([None] * 12), 4096 + 8, 1 << 30, None) == 5
    assert lib.swimba_mixer_fwd(ctypes.byref(d), *([None] * 12), 4096, 16, None) == 5
    # aligned and large enough workspace, but tensor pointers missing
    assert lib.swimba_mixer_fwd(ctypes.byref(d), *([None] * 12), 4096, 1 << 30, None) == 1
    # step: seqlen must be 1; then NULL pointers
    assert lib.swimba_step(ctypes.byref(d), *([None] * 11), None, 0, None) == 2
    d1 = dims(seqlen=1)
    assert lib.swimba_step(ctypes.byref(d1), *([None] * 11), None, 0, None) == 5
    assert sw.swimba_step_workspace_bytes(d1) >= 1 * 1 * 16 * 2 * 4 and sw.swimba_step_workspace_bytes(d) == 0
    assert lib.swimba_step(ctypes.byref(d1), *([None] * 11), 4096, 1 << 20, None) == 1
    assert lib.swimba_router_topk(10, 4, 5, 0, None, None, None, None) == 2
    assert lib.swimba_router_topk(10, 4, 2, 0, None, None, None, None) == 1
    assert lib.swimba_router_topk(0, 4, 2, 0, None, None, None, None) == 0
    assert lib.swimba_probe_copy(None, None, 16, None) == 1
    assert lib.swimba_status_string(4).decode().startswith("problem outside")
    assert lib.swimba_last_hip_error() == 0


def test_misaligned_pointers_are_refused_on_the_host():
    """Pointer values only (never dereferenced: a refused call enqueues nothing).  Large tensors
    need 16 bytes, per-token and per-head tensors the alignment of their elements."""
    lib = sw._load()
    d = dims()
    ok = [0x10000 * (i + 1) for i in range(12)]    # x dt A D Be Ce logits h0 y h_final topk_idx topk_w
    ws, wsb = 0x4000000, 1 << 30
    for pos, off in [(0, 8), (4, 4), (5, 2), (8, 8), (7, 4), (9, 12),      # 16-byte tensors
                     (1, 2), (6, 1), (2, 2), (10, 2), (11, 1)]:            # element alignment (fp32 io: 4 bytes)
        args = list(ok)
        args[pos] += off
        assert lib.swimba_mixer_fwd(ctypes.byref(d), *args, ws, wsb, None) == 7, (pos, off)
    # bf16 io: dt and logits need 2 bytes only -> refused at 1, and the big tensors still need 16
    db = dims(io_dtype=1)
    args = list(ok); args[1] += 1
    assert lib.swimba_mixer_fwd(ctypes.byref(db), *args, ws, wsb, None) == 7
    args = list(ok); args[0] += 2
    assert lib.swimba_mixer_fwd(ctypes.byref(db), *args, ws, wsb, None) == 7
    # decode step and router
    d1 = dims(seqlen=1)
    sargs = [0x10000 * (i + 1) for i in range(11)]  # state_in state_out x dt A D Be Ce logits y topk_idx
    sargs[0] += 4
    assert lib.swimba_step(ctypes.byref(d1), *sargs, ws, 1 << 20, None) == 7
    assert lib.swimba_router_topk(10, 4, 2, 0, 0x10002, 0x20000, 0x30000, None) == 7
    assert lib.swimba_status_string(7).decode().startswith("a tensor pointer is not aligned")


def test_later_entry_points_validate_on_the_host():
    """Separated, expert-X, projection, selected-stream and multi-token entry points: invalid dims,
    missing workspace, NULL and misaligned pointers are all refused before anything is enqueued."""
    lib = sw._load()
    d = dims()
    big = 1 << 30
    ws = 0x4000000
    p = [0x10000 * (i + 1) for i in range(16)]
    # workspace queries: positive for valid dims, 0 for invalid ones
    for q in (sw.swimba_separated_workspace_bytes, sw.swimba_mixer_xe_workspace_bytes):
        assert q(d) >= sw.swimba_mixer_workspace_bytes(d) and q(dims(top_k=9)) == 0
    assert sw.swimba_expert_proj_workspace_bytes(d, 64) > 0 and sw.swimba_expert_proj_workspace_bytes(d, 0) == 0
    assert sw.swimba_mixer_proj_workspace_bytes(d, 64) > sw.swimba_mixer_workspace_bytes(d)
    assert sw.swimba_mixer_proj_workspace_bytes(dims(chunk=0), 64) == 0
    # separated: (dims, x dt A D Be Ce logits y idx w, ws, bytes, stream)
    assert lib.swimba_separated_fwd(ctypes.byref(dims(ngroups=3)), *p[:10], ws, big, None) == 2
    assert lib.swimba_separated_fwd(ctypes.byref(d), *p[:10], None, 0, None) == 5
    assert lib.swimba_separated_fwd(ctypes.byref(d), None, *p[1:10], ws, big, None) == 1
    assert lib.swimba_separated_fwd(ctypes.byref(d), p[0] + 8, *p[1:10], ws, big, None) == 7
    # expert-X: (dims, xe dt A D Be Ce logits h0 y h_final idx w, ws, bytes, stream)
    assert lib.swimba_mixer_fwd_xe(ctypes.byref(d), *p[:12], ws, 16, None) == 5
    assert lib.swimba_mixer_fwd_xe(ctypes.byref(d), *p[:5], None, *p[6:12], ws, big, None) == 1
    assert lib.swimba_mixer_fwd_xe(ctypes.byref(d), *p[:8], p[8] + 4, *p[9:12], ws, big, None) == 7
    # projection, dense and per selected slot: (dims, d_model, u WB WC logits Bo Co idx w, ws, bytes, stream)
    for fn in (lib.swimba_expert_proj, lib.swimba_expert_proj_selected):
        assert fn(ctypes.byref(d), 0, *p[:8], ws, big, None) == 2
        assert fn(ctypes.byref(d), 64, *p[:8], ws + 64, big, None) == 5
        assert fn(ctypes.byref(d), 64, *p[:2], None, *p[3:8], ws, big, None) == 1
        assert fn(ctypes.byref(d), 64, *p[:4], p[4] + 2, *p[5:8], ws, big, None) == 7
        # outside the MFMA GEMM's shapes (here fp32 io) one token's features sit in LDS: width limit
        assert fn(ctypes.byref(d), 16400, *p[:8], ws, big, None) == 4
    assert sw.swimba_expert_proj_workspace_bytes(d, 16384) > 0 and sw.swimba_expert_proj_workspace_bytes(d, 16400) == 0
    # the GEMM's shapes (bf16, d_model % 16 == 0, (G*N) % 64 == 0) take up to 65536 features
    dg = dims(io_dtype=1, dstate=64)
    assert sw.swimba_expert_proj_workspace_bytes(dg, 65536) > 0 and sw.swimba_expert_proj_workspace_bytes(dg, 65552) == 0
    assert sw.swimba_expert_proj_workspace_bytes(dg, 16392) == 0       # not a multiple of 16: generic kernel
    assert sw.swimba_mixer_proj_workspace_bytes(d, 16400) == 0
    # forward on selected streams: (dims, x dt A D Bsel Csel w h0 y h_final, ws, bytes, stream)
    assert lib.swimba_mixer_fwd_selected(ctypes.byref(d), *p[:10], None, 0, None) == 5
    assert lib.swimba_mixer_fwd_selected(ctypes.byref(d), *p[:6], None, *p[7:10], ws, big, None) == 1
    assert lib.swimba_mixer_fwd_selected(ctypes.byref(d), *p[:6], p[6] + 2, *p[7:10], ws, big, None) == 7
    # projection + forward: (dims, d_model, u WB WC x dt A D logits h0 y h_final idx w, ws, bytes, stream)
    assert lib.swimba_mixer_fwd_proj(ctypes.byref(d), 64, *p[:13], ws, 1024, None) == 5
    assert lib.swimba_mixer_fwd_proj(ctypes.byref(d), 64, None, *p[1:13], ws, big, None) == 1
    assert lib.swimba_mixer_fwd_proj(ctypes.byref(d), 64, *p[:3], p[3] + 8, *p[4:13], ws, big, None) == 7
    assert lib.swimba_mixer_fwd_proj(ctypes.byref(dims(headdim=128, dstate=128)), 64, *p[:13], ws, big, None) == 4
    # router linear map: (tokens, d_model, nexperts, io_dtype, u, W_g, logits, stream)
    assert lib.swimba_router_linear(10, 0, 4, 0, p[0], p[1], p[2], None) == 2
    assert lib.swimba_router_linear(10, 16, 300, 0, p[0], p[1], p[2], None) == 4
    assert lib.swimba_router_linear(10, 16, 4, 5, p[0], p[1], p[2], None) == 3
    assert lib.swimba_router_linear(10, 16, 4, 0, p[0], None, p[2], None) == 1
    assert lib.swimba_router_linear(10, 16, 4, 1, p[0] + 8, p[1], p[2], None) == 7
    assert lib.swimba_router_linear(0, 16, 4, 1, None, None, None, None) == 0
    # several decode tokens per call: at most 64, at least 1
    assert sw.swimba_step_multi_workspace_bytes(dims(seqlen=65)) == 0
    assert lib.swimba_step_multi(ctypes.byref(dims(seqlen=65)), *p[:11], ws, big, None) == 4
    assert lib.swimba_step_multi(ctypes.byref(dims(seqlen=4)), *p[:11], None, 0, None) == 5
    assert lib.swimba_step_multi(ctypes.byref(dims(seqlen=4)), *p[:2], None, *p[3:11], ws, big, None) == 1
    assert lib.swimba_step_multi(ctypes.byref(dims(seqlen=4)), *p[:9], p[9] + 8, p[10], ws, big, None) == 7


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/swimba.h compiles as C99 with gcc (no C++ in the boundary), and a C program that
    only uses host-side calls links against libswimba.so and runs without a GPU."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "abi.c"
    src.write_text(
        '#include "swimba.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "  swimba_dims d = {1, 256, 4, 16, 16, 1, 4, 2, 64, SWIMBA_F32};\n"
        "  size_t n = swimba_mixer_workspace_bytes(&d);\n"
        "  swimba_ws_layout lo;\n"
        "  if (swimba_mixer_workspace_layout(&d, &lo) != SWIMBA_OK || lo.total != n || n == 0) return 1;\n"
        "  if (swimba_mixer_fwd(&d, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) != SWIMBA_ERR_WORKSPACE) return 2;\n"
        '  printf("%s\\n", swimba_status_string(SWIMBA_ERR_ALIGNMENT));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "abi"
    libdir = os.path.join(root, "paper_2603_06938_amd")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                        str(src), "-o", str(exe), "-L", libdir, "-l:libswimba.so", "-Wl,-rpath," + libdir],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert "aligned" in r.stdout


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 4, 2, 16)
    Be = torch.zeros(1, 4, 3, 1, 16)
    with pytest.raises((ValueError, sw.SwimbaError)):
        sw.swimba_mixer_fwd(x, torch.ones(1, 4, 2), -torch.ones(2), None, Be, Be, torch.zeros(1, 4, 3),
                            2, 4, workspace=torch.zeros(1 << 16, dtype=torch.uint8))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
