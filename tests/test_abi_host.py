"""Host-side checks of the C ABI: the library loads, exports what include/lawcat.h declares,
and every argument error is reported before anything touches a GPU.  CPU only."""
import ctypes
import os
import re

import pytest

from paper_2509_18467_amd import lawcat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "lawcat.h")).read()
    declared = re.findall(r"LAWCAT_API\s+[\w\s\*]+?\b(lawcat_\w+)\s*\(", text)
    assert sorted(declared) == sorted(lawcat.EXPORTS)
    L = lawcat.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert lawcat.version() == 1


def test_desc_matches_header_layout():
    assert ctypes.sizeof(lawcat.Desc) == 15 * 4
    text = open(os.path.join(ROOT, "include", "lawcat.h")).read()
    body = re.search(r"typedef struct lawcat_desc \{(.*?)\} lawcat_desc;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            names += [n.strip() for n in decl.split(None, 1)[1].split(",")]
    assert names == [f[0] for f in lawcat.Desc._fields_]


A = ctypes.c_void_p(0x1000)  # fake, 16-byte aligned device address: never dereferenced on error paths


def _layer(desc, **over):
    args = dict(Q=A, K=A, V=A, G=A, wq=A, wk=A, S0=None, z0=None, qh=None, kh=None, O=A, den=None, S=A, z=A,
                qt=None, kt=None, ws=A, wsb=1 << 40, stream=None)
    args.update(over)
    return lawcat.lib().lawcat_layer_prefill(ctypes.byref(desc), *args.values())


def test_null_and_bad_desc():
    L = lawcat.lib()
    assert L.lawcat_layer_prefill(None, *([None] * 17), 0, None) == -1
    d = lawcat.make_desc(1, 256, 2, 2, 64, dtype=0)
    assert _layer(d, Q=None) == -1
    assert _layer(d, S=None) == -1
    bad = lawcat.make_desc(1, 256, 2, 2, 64)
    bad.struct_size = 8
    assert _layer(bad) == -2
    assert _layer(lawcat.make_desc(1, 0, 2, 2, 64)) == -2
    assert _layer(lawcat.make_desc(1, 16, 3, 2, 64)) == -2
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, dtype=7)) == -2
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, feature_map=2)) == -2
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, carry_mode=3)) == -2
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, gate_scale=float("nan"))) == -2
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, gate_scale=-1.0)) == -2


def test_unsupported_shapes():
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 48)) == -3
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, conv_width=5)) == -3
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, chunk=64)) == -3
    assert _layer(lawcat.make_desc(1, 16, 2, 2, 64, segment=100)) == -3
    d = lawcat.make_desc(1, 16, 2, 2, 64)
    d.dv = 128
    assert _layer(d) == -3


def test_alignment_and_workspace():
    d = lawcat.make_desc(1, 256, 2, 2, 64, dtype=0)
    assert _layer(d, K=ctypes.c_void_p(0x1008)) == -5
    need = lawcat.workspace_bytes(d, lawcat.CALL_LAYER_PREFILL)
    assert need >= 256 * 4 * 64 * 4
    assert _layer(d, ws=None) == -4
    assert _layer(d, wsb=need - 1) == -4
    assert lawcat.workspace_bytes(d, lawcat.CALL_CONV1D) == 0
    assert lawcat.workspace_bytes(d, lawcat.CALL_GLA_STEP) == 0
    assert lawcat.workspace_bytes(lawcat.make_desc(1, 16, 3, 2, 64), lawcat.CALL_LAYER_PREFILL) == 0


def test_path_selection_shows_in_workspace_size():
    """Shapes the matrix-core path does not take fall back to the unfused fp32-accumulating path, whose
    workspace holds q-dot and k-dot: rows that need more than 32-bit byte offsets, more (batch, kv head)
    pairs than a grid axis holds, more than 64 query heads per kv head."""
    def unfused(B, T, Hq, Hkv, d):
        up = lambda n: (n + 255) // 256 * 256
        return up(B * T * Hq * d * 2) + up(B * T * Hkv * d * 2)

    call = lawcat.CALL_LAYER_PREFILL
    ok = lawcat.make_desc(1, 32768, 32, 8, 64)
    assert 0 < lawcat.workspace_bytes(ok, call) < 32 * 1024 * 1024  # segment states only
    long_rows = lawcat.make_desc(1, 1 << 20, 32, 8, 64)             # 2^20 tokens x 4 KiB rows = 4 GiB
    assert lawcat.workspace_bytes(long_rows, call) == unfused(1, 1 << 20, 32, 8, 64)
    # the last granule's rows past T must not wrap a 32-bit offset either: the limit sits 128 rows below 4 GiB
    near = lawcat.make_desc(1, (1 << 20) - 64, 32, 8, 64)
    assert lawcat.workspace_bytes(near, call) == unfused(1, (1 << 20) - 64, 32, 8, 64)
    below = lawcat.make_desc(1, (1 << 20) - 129, 32, 8, 64)
    assert 0 < lawcat.workspace_bytes(below, call) < 64 * 1024 * 1024
    many_heads = lawcat.make_desc(70000, 16, 1, 1, 64)
    assert lawcat.workspace_bytes(many_heads, call) == unfused(70000, 16, 1, 1, 64)
    group8 = lawcat.make_desc(1, 4096, 16, 2, 64)   # covered by two launches over 4 query heads each
    assert 0 < lawcat.workspace_bytes(group8, call) < unfused(1, 4096, 16, 2, 64)
    group65 = lawcat.make_desc(1, 4096, 130, 2, 64)
    assert lawcat.workspace_bytes(group65, call) == unfused(1, 4096, 130, 2, 64)


def test_other_entry_points_report_errors():
    L = lawcat.lib()
    d = lawcat.make_desc(2, 64, 4, 2, 128)
    r = ctypes.byref(d)
    assert L.lawcat_conv1d_causal(r, 0, A, A, None, A, None, None) == -2
    assert L.lawcat_conv1d_causal(r, 4, None, A, None, A, None, None) == -1
    assert L.lawcat_conv1d_causal(r, 4, A, A, ctypes.c_void_p(0x1004), A, None, None) == -5
    assert L.lawcat_gla_prefill(r, A, A, A, None, None, None, A, None, A, A, A, 1 << 40, None) == -1
    assert L.lawcat_gla_prefill(r, A, A, A, A, None, None, A, None, A, None, A, 1 << 40, None) == -1
    assert L.lawcat_gla_step(r, A, A, A, A, None, A, A, None) == -1
    d0 = lawcat.make_desc(2, 0, 4, 2, 128)  # T is ignored by the step, checked by prefill
    assert L.lawcat_gla_step(ctypes.byref(d0), A, A, A, A, A, ctypes.c_void_p(0x1001), A, None) == -5
    assert L.lawcat_gla_prefill(ctypes.byref(d0), A, A, A, A, None, None, A, None, A, A, A, 1 << 40, None) == -2


def test_status_strings():
    seen = {lawcat.status_string(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and "unknown status" not in seen
    assert lawcat.status_string(-99) == "unknown status"
    with pytest.raises(lawcat.LawcatError):
        lawcat._check(-3)


def test_gla_steps_argument_checks():
    L = lawcat.lib()
    d = lawcat.make_desc(1, 8, 4, 2, 64)
    ok = [A] * 7
    assert L.lawcat_gla_steps(None, *ok, None) == -1
    assert L.lawcat_gla_steps(ctypes.byref(d), None, *ok[1:], None) == -1
    assert L.lawcat_gla_steps(ctypes.byref(d), *ok[:4], None, A, A, None) == -1
    assert L.lawcat_gla_steps(ctypes.byref(d), ctypes.c_void_p(0x1004), *ok[1:], None) == -5
    assert L.lawcat_gla_steps(ctypes.byref(lawcat.make_desc(1, 0, 4, 2, 64)), *ok, None) == -2
    assert L.lawcat_gla_steps(ctypes.byref(lawcat.make_desc(1, 8, 4, 2, 96)), *ok, None) == -3


def test_static_entry_point_rejects_what_its_buffer_cannot_hold():
    """lawcat_layer_prefill_static checks the desc and the scratch need before anything else."""
    L = lawcat.lib()

    def static(desc, Q=A):
        return L.lawcat_layer_prefill_static(ctypes.byref(desc), Q, A, A, A, A, A, None, None, None, None, A, None, A,
                                             A, None, None, None)

    big = lawcat.make_desc(4, 131072, 32, 8, 128, segment=1024)   # 32 heads x 128 segment states of 65 KiB
    assert lawcat.workspace_bytes(big, lawcat.CALL_LAYER_PREFILL) > lawcat.STATIC_WORKSPACE_BYTES
    assert static(big) == -7
    fp32_long = lawcat.make_desc(1, 32768, 32, 8, 64, dtype=0)   # fp32 storage stages q-dot and k-dot: 320 MiB
    assert static(fp32_long) == -7
    assert static(lawcat.make_desc(1, 0, 2, 2, 64)) == -2
    assert static(lawcat.make_desc(1, 4096, 32, 8, 64), Q=None) == -1
    assert "static buffer" in lawcat.status_string(-7)
    text = open(os.path.join(ROOT, "include", "lawcat.h")).read()
    assert int(re.search(r"LAWCAT_STATIC_WORKSPACE_BYTES \((\d+)u << 20\)", text).group(1)) << 20 == lawcat.STATIC_WORKSPACE_BYTES


def test_feature_map_entry_points_check_their_arguments():
    """lawcat_conv1d_feature and lawcat_layer_prefill_fm: shared matrix required, head count a multiple of Hkv,
    workspace = staged q-dot and k-dot plus what lawcat_gla_prefill needs."""
    L = lawcat.lib()
    d = lawcat.make_desc(1, 4096, 32, 8, 64)

    def feat(desc, n_heads, wf=A, x=A):
        return L.lawcat_conv1d_feature(ctypes.byref(desc), n_heads, x, A, wf, None, A, None, None)

    assert feat(d, 32, wf=None) == -1
    assert feat(d, 12) == -2                      # 12 query heads cannot share 8 matrices evenly
    assert feat(d, 0) == -2
    assert feat(d, 8, x=ctypes.c_void_p(0x1004)) == -5
    assert feat(lawcat.make_desc(1, 16, 4, 2, 96), 4) == -3

    need = lawcat.workspace_bytes(d, lawcat.CALL_LAYER_PREFILL_FM)
    staged = 4096 * (32 + 8) * 64 * 2
    assert need >= staged + lawcat.workspace_bytes(d, lawcat.CALL_GLA_PREFILL)
    assert need < staged + lawcat.workspace_bytes(d, lawcat.CALL_GLA_PREFILL) + 3 * 256
    f32 = lawcat.make_desc(1, 512, 4, 2, 64, dtype=0)
    assert lawcat.workspace_bytes(f32, lawcat.CALL_LAYER_PREFILL_FM) >= 512 * 6 * 64 * 4

    def layer(desc, ws, nbytes, wf=A):
        return L.lawcat_layer_prefill_fm(ctypes.byref(desc), A, A, A, A, A, A, wf, None, None, None, None, A, None,
                                         A, A, None, None, ws, nbytes, None)

    assert layer(d, A, need, wf=None) == -1
    assert layer(d, A, need - 1) == -4
    assert layer(d, None, 0) == -4
    assert layer(lawcat.make_desc(1, 0, 4, 2, 64), A, need) == -2


def test_varlen_entry_point_checks_every_sequence_first():
    """lawcat_layer_prefill_varlen: offsets start at 0 and increase strictly, no length above desc.T, workspace
    enough for the longest sequence -- all before anything is enqueued."""
    L = lawcat.lib()
    d = lawcat.make_desc(3, 4096, 32, 8, 64)

    def call(starts, desc=d, ws=A, nbytes=1 << 30, den=None, Q=A, dev=None):
        arr = (ctypes.c_int32 * len(starts))(*starts)
        return L.lawcat_layer_prefill_varlen(ctypes.byref(desc), arr, dev, Q, A, A, A, A, A, None, None, None, None, A, den,
                                             A, A, None, None, ws, nbytes, None)

    assert call([1, 100, 200, 300]) == -2          # must start at 0
    assert call([0, 100, 100, 300]) == -2          # empty sequence
    assert call([0, 100, 50, 300]) == -2           # decreasing
    assert call([0, 100, 200, 4500]) == -2         # longer than desc.T
    assert call([0, 100, 200, 300], Q=None) == -1
    assert call([0, 4096, 8192, 8292], ws=None, nbytes=0) == -4
    need = lawcat.varlen_workspace_bytes(d, [0, 4096, 8192, 8292])
    assert need == lawcat.workspace_bytes(lawcat.make_desc(1, 4096, 32, 8, 64), lawcat.CALL_LAYER_PREFILL) > 0
    assert call([0, 4096, 8192, 8292], nbytes=need - 1) == -4
    assert call([0, 100, 200, 300], den=ctypes.c_void_p(0x1004)) == -5
    # with a device copy of the offsets the batch is one set of launches: workspace as for B sequences of desc.T tokens
    assert call([0, 100, 200, 4500], dev=A) == -2
    assert call([0, 100, 200, 300], dev=ctypes.c_void_p(0x1002)) == -5
    whole = lawcat.varlen_workspace_bytes(d, [0, 4096, 8192, 8292], one_launch=True)
    assert whole > 0 and call([0, 4096, 8192, 8292], dev=A, nbytes=whole - 1) == -4
    # segments are cut as for one sequence of all 8292 tokens (512 workgroups wanted, 8 kv heads: 64 per head,
    # 192 tokens each: 22 + 22 + 1 segments = 360 workgroups, they fit), slots laid out for the longest sequence:
    # 3 sequences x 8 heads x ceil(4096 / 192) slots
    slot = (64 * 64 + 2 * 64) * 4 + 4
    assert whole == 3 * 8 * 22 * slot
    assert lawcat.varlen_workspace_bytes(d, [0, 4097, 8192, 9000]) == 0     # a length above desc.T


def test_gate_project_argument_checks():
    L = lawcat.lib()
    d = lawcat.make_desc(1, 4096, 32, 8, 64)

    def call(dm=2048, rank=32, x=A, bias=None, desc=d):
        return L.lawcat_gate_project(ctypes.byref(desc), dm, rank, x, A, A, bias, A, None)

    assert call(x=None) == -1
    assert call(dm=0) == -2 and call(rank=0) == -2
    assert call(dm=2047) == -3 and call(rank=12) == -3
    assert call(dm=16384) == -3                     # a row of x plus the intermediate must fit 64 KB of LDS as fp32
    assert call(bias=ctypes.c_void_p(0x1008)) == -5
    assert call(desc=lawcat.make_desc(1, 0, 32, 8, 64)) == -2


def test_gla_backward_argument_checks():
    L = lawcat.lib()
    d = lawcat.make_desc(1, 4096, 32, 8, 64)
    need = lawcat.workspace_bytes(d, lawcat.CALL_GLA_BACKWARD)
    # dden and the gate term per token in fp32; two sets of segment states and the gate totals for 8 kv heads x 64
    # segments of 64 tokens (about 1024 workgroups wanted)
    assert need == 4 * (4096 * (32 + 8 * 64) + 8 * 64 * (2 * (64 * 64 + 128) + 64)) + 256

    def call(desc=d, q=A, den=A, dO=A, dq=A, dS0=None, ws=A, nbytes=need):
        return L.lawcat_gla_backward(ctypes.byref(desc), q, A, A, A, den, dO, None, None, dq, A, A, A, dS0, None,
                                     ws, nbytes, None)

    assert call(q=None) == -1 and call(den=None) == -1 and call(dO=None) == -1 and call(dq=None) == -1
    assert call(dS0=ctypes.c_void_p(0x1004)) == -5
    assert call(ws=None) == -4 and call(nbytes=need - 1) == -4
    assert call(desc=lawcat.make_desc(1, 0, 32, 8, 64)) == -2
    assert call(desc=lawcat.make_desc(1, 4096, 64, 2, 128)) == -3     # 32 query heads of 128 per kv head: staging too large
    assert lawcat.workspace_bytes(lawcat.make_desc(1, 4096, 32, 8, 128), lawcat.CALL_GLA_BACKWARD) > need


def test_conv1d_backward_argument_checks():
    L = lawcat.lib()
    d = lawcat.make_desc(2, 1000, 32, 8, 64)
    need = lawcat.workspace_bytes(d, lawcat.CALL_CONV1D_BACKWARD)
    assert need == 2 * 16 * 32 * 64 * 4 * 4          # (batch, 64-token strip) partial sums of dw [Hq, d, W] in fp32

    def call(desc=d, heads=32, x=A, dy=A, dw=A, dhalo=None, ws=A, nbytes=need):
        return L.lawcat_conv1d_backward(ctypes.byref(desc), heads, x, A, None, dy, A, dw, dhalo, ws, nbytes, None)

    assert call(x=None) == -1 and call(dy=None) == -1 and call(dw=None) == -1
    assert call(heads=0) == -2
    assert call(dhalo=ctypes.c_void_p(0x1008)) == -5
    assert call(ws=None) == -4 and call(nbytes=need - 1) == -4
    assert call(heads=8, nbytes=need // 4 - 1) == -4             # the key conv needs a quarter of it
    assert call(desc=lawcat.make_desc(2, 1000, 32, 8, 64, conv_width=5)) == -3


def test_packed_batch_plan_fits_the_chip_in_one_round():
    """The one-launch plan of a packed batch: the workspace grows with the longest sequence only through its segment
    count, many short sequences get one segment each, and lengthening the segments keeps the workgroups within
    the 512 (head dim 64) or 256 (128) the chip holds at once -- read off the workspace size, which is
    sequences x kv heads x segments-of-the-longest x slot bytes."""
    def slots_of(d, starts, **kw):
        desc = lawcat.make_desc(len(starts) - 1, max(b - a for a, b in zip(starts, starts[1:])), 32, 8, d, **kw)
        need = lawcat.varlen_workspace_bytes(desc, starts, one_launch=True)
        slot = (d * d + 2 * d) * 4 + 4
        assert need % ((len(starts) - 1) * 8 * slot) == 0
        return need // ((len(starts) - 1) * 8 * slot)        # segments of the longest sequence (0: one segment each)

    def cum(lengths):
        out = [0]
        for n in lengths:
            out.append(out[-1] + n)
        return out

    # 24 sequences, 32768 tokens: 512-token segments would give 544 workgroups; 640-token ones give 512
    mix = [4096, 2048, 1024, 512, 256, 256] * 4
    assert slots_of(64, cum(mix)) == 7                        # ceil(4096 / 640)
    # one long sequence behaves as lawcat_layer_prefill does
    assert slots_of(64, [0, 32768]) == 64
    # 100 short sequences: more (sequence, head) pairs than places, one segment each, no workspace
    assert slots_of(64, cum([300] * 100)) == 0
    # head dim 128: 256 places
    assert slots_of(128, [0, 16384]) == 32
    # an explicit segment length is taken as given
    assert slots_of(64, cum(mix), segment=256) == 16
