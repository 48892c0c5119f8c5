"""The C-ABI library loads without a GPU, exports every symbol include/idlm.h declares, and
rejects bad host-visible arguments before touching the device (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

import paper_2604_11035_amd as idlm

INCLUDE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
HEADERS = sorted(os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h"))


def declared_functions(headers=None):
    names = set()
    for h in headers or HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(idlm_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"idlm_isd_attention", "idlm_isd_accept", "idlm_isd_attention_workspace",
            "idlm_isd_accept_workspace", "idlm_strerror", "idlm_version"} <= set(names)
    L = idlm.lib()
    for n in names:
        assert getattr(L, n) is not None, n
    # the method's header holds the step's calls only; timing hooks, byte-counter calibration and the
    # generator dump are declared apart
    main = set(declared_functions([os.path.join(INCLUDE, "idlm.h")]))
    aids = set(declared_functions([os.path.join(INCLUDE, "idlm_debug.h")])) - main
    assert aids == {"idlm_isd_attention_ev", "idlm_isd_accept_ev", "idlm_isd_accept_bf16_ev", "idlm_isd_rng_dump",
                    "idlm_isd_attention_wave_trace", "idlm_stream_copy", "idlm_stream_read"}
    assert not any(n.endswith("_ev") or n.startswith("idlm_stream") for n in main)


def test_version_and_error_strings():
    assert idlm.idlm_version() == 202
    seen = set()
    for code in range(0, -8, -1):
        msg = idlm.idlm_strerror(code)
        assert msg and msg not in seen
        seen.add(msg)
    assert "unknown" in idlm.idlm_strerror(-99)


def test_workspace_sizes_are_host_only_and_monotone():
    a = idlm.idlm_isd_accept_workspace(256, 16, 151936)
    b = idlm.idlm_isd_accept_workspace(16, 8, 32768)
    assert a > b > 0 and a % 256 == 0
    assert idlm.idlm_isd_accept_workspace(4, 4, 1023) == 0          # V % 4 != 0 is rejected
    assert idlm.idlm_isd_accept_workspace(4, 65, 1024) == 0
    w = idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 1)
    assert w > 0
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 2) == w   # operand-order K pages: same kernels
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 0) == 0   # fp32 path needs none
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 64, 16, 512, 1) == 2 * 256 * 4 * 4 * (4 * 64 * 8 + 16 * 16)   # D = 64: half-size rows
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 64, 16, 512, 2) == 0    # operand-order K pages exist for D = 128 only
    assert idlm.idlm_isd_attention_workspace(256, 33, 32, 8, 128, 16, 512, 1) == 0
    # sized by the grid that will be launched: two slots of 64 rows (17 KB) per wavefront
    assert w == 2 * 256 * 4 * 4 * (4 * 64 * 16 + 16 * 16)
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 1, 1024) == 4 * w
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 1, 64) == w // 4
    assert idlm.idlm_isd_attention_workspace(256, 4, 32, 8, 128, 16, 512, 1) == w // 4      # 16 rows per KV head
    assert idlm.idlm_isd_attention_workspace(256, 16, 32, 8, 128, 16, 512, 1, 1025) == 0


FAKE = C.c_void_p(0x1000)        # non-NULL, 16-byte aligned, never dereferenced (validation only)
ODD = C.c_void_p(0x1004)


def _attention(**kw):
    a = dict(q=FAKE, k=FAKE, v=FAKE, table=FAKE, ctx=FAKE, S=4, out=FAKE, B=2, Hq=8, Hkv=2, D=128, P=16,
             num_pages=10, max_pages=4, ps=2 * 16 * 128, hs=16 * 128, ts=128, scale=0.0, dtype=1, nwg=0,
             ws=None, ws_bytes=0, stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_attention(a["q"], a["k"], a["v"], a["table"], a["ctx"], a["S"], a["out"], a["B"],
                                         a["Hq"], a["Hkv"], a["D"], a["P"], a["num_pages"], a["max_pages"],
                                         a["ps"], a["hs"], a["ts"], a["scale"], a["dtype"], a["nwg"], a["ws"],
                                         a["ws_bytes"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(q=None), -1), (dict(out=None), -1), (dict(table=None), -1),
    (dict(S=0), -2), (dict(S=33), -2), (dict(Hq=7), -2), (dict(P=32), -2), (dict(max_pages=0), -2),
    (dict(S=32, Hq=32, Hkv=2), -2),            # S*G = 512 rows
    (dict(nwg=-1), -2), (dict(nwg=5000), -2), (dict(ts=64), -2),
    (dict(dtype=7), -3), (dict(D=96), -3), (dict(D=96, dtype=0), -3),
    (dict(dtype=2, D=64), -3), (dict(dtype=2, ts=256, hs=128, ps=16 * 256), -3),   # operand-order K pages need D = token_stride = 128
    (dict(q=ODD), -4), (dict(k=ODD), -4), (dict(ts=132), -4),
    (dict(), -5),                              # bf16 path without a workspace
    (dict(dtype=2), -5),                       # operand-order K pages: the same path
    (dict(ws=FAKE, ws_bytes=16), -5),
])
def test_attention_rejects_bad_arguments(kw, code):
    assert _attention(**kw) == code


def test_attention_empty_batch_is_ok_without_device():
    assert _attention(B=0) == 0


def _accept(**kw):
    a = dict(logits=FAKE, drafts=FAKE, seed=1, alen=FAKE, toks=FAKE, B=2, S=4, V=1024, ndu=1, nd=None,
             greedy=None, off=0, probs=None, ws=None, ws_bytes=0, stream=None)
    a.update(kw)
    fn = getattr(idlm.lib(), a.pop("fn", "idlm_isd_accept"))
    return fn(a["logits"], a["drafts"], a["seed"], a["alen"], a["toks"], a["B"], a["S"], a["V"], a["ndu"], a["nd"],
              a["greedy"], a["off"], a["probs"], a["ws"], a["ws_bytes"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(logits=None), -1), (dict(alen=None), -1), (dict(toks=None), -1), (dict(drafts=None), -1),
    (dict(S=0), -2), (dict(S=65), -2), (dict(V=1022), -2), (dict(V=0), -2), (dict(ndu=4), -2), (dict(ndu=-1), -2),
    (dict(logits=ODD), -4),
    (dict(), -5), (dict(ws=FAKE, ws_bytes=8), -5),
])
def test_accept_rejects_bad_arguments(kw, code):
    assert _accept(**kw) == code


@pytest.mark.parametrize("kw,code", [
    (dict(logits=None), -1), (dict(alen=None), -1), (dict(toks=None), -1), (dict(drafts=None), -1),
    (dict(S=0), -2), (dict(S=65), -2), (dict(V=1028), -2), (dict(V=4), -2), (dict(V=0), -2), (dict(ndu=4), -2),
    (dict(logits=ODD), -4),
    (dict(), -5), (dict(ws=FAKE, ws_bytes=8), -5), (dict(B=0), 0),
])
def test_accept_bf16_rejects_bad_arguments(kw, code):
    assert _accept(fn="idlm_isd_accept_bf16", **kw) == code


def test_accept_empty_batch_and_single_row_without_drafts():
    assert _accept(B=0) == 0
    # S = 1 needs no draft array: gets past the NULL checks and stops at the missing workspace
    assert _accept(S=1, ndu=0, drafts=None) == -5


def test_accept_static_checks_shapes_and_its_fixed_limit_before_touching_a_device():
    L = idlm.lib()
    cap = idlm.idlm_isd_accept_static_max_bytes()
    assert cap == 1 << 20 and idlm.idlm_isd_accept_workspace(256, 16, 151936) < cap

    def call(B=2, S=4, V=1024, ndu=1):
        return L.idlm_isd_accept_static(FAKE, FAKE, 7, FAKE, FAKE, B, S, V, ndu, None, None, 0, None, None)
    assert call(B=0) == 0
    assert call(S=0) == -2 and call(S=65) == -2 and call(V=1023) == -2 and call(B=-1) == -2
    assert idlm.idlm_isd_accept_workspace(8192, 16, 1024) > cap
    assert call(B=8192, S=16) == -5                      # beyond the fixed array: refused, nothing launched


def test_stream_helpers_validate():
    L = idlm.lib()
    assert L.idlm_stream_copy(None, FAKE, 16, None) == -1
    assert L.idlm_stream_copy(FAKE, FAKE, 10, None) == -2
    assert L.idlm_stream_copy(ODD, FAKE, 16, None) == -4
    assert L.idlm_stream_copy(FAKE, FAKE, 0, None) == 0
    assert L.idlm_stream_read(FAKE, 32, None, None) == -1


def _append(**kw):
    a = dict(kn=FAKE, vn=FAKE, kc=FAKE, vc=FAKE, table=FAKE, ctx=FAKE, S=4, B=2, Hkv=2, D=128, P=16, num_pages=10,
             max_pages=4, ps=2 * 16 * 128, hs=16 * 128, ts=128, dtype=1, stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_kv_append(a["kn"], a["vn"], a["kc"], a["vc"], a["table"], a["ctx"], a["S"], a["B"],
                                         a["Hkv"], a["D"], a["P"], a["num_pages"], a["max_pages"], a["ps"], a["hs"],
                                         a["ts"], a["dtype"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(kn=None), -1), (dict(vc=None), -1), (dict(ctx=None), -1),
    (dict(S=0), -2), (dict(S=65), -2), (dict(B=70000), -2), (dict(num_pages=0), -2), (dict(ts=64), -2),
    (dict(dtype=5), -3), (dict(dtype=2, D=64, ts=64), -3), (dict(dtype=2, ts=256), -3), (dict(dtype=2, P=32), -3),
    (dict(kn=ODD), -4), (dict(kc=ODD), -4), (dict(D=4), -4), (dict(ts=132), -4),
])
def test_kv_append_rejects_bad_arguments(kw, code):
    assert _append(**kw) == code


def test_kv_append_empty_batch_is_ok_without_device():
    assert _append(B=0) == 0


def _commit(**kw):
    a = dict(alen=FAKE, toks=FAKE, nd=FAKE, ctx=FAKE, stride=FAKE, drafts=FAKE, out=FAKE, olen=FAKE, cap=32,
             table=FAKE, used=FAKE, free=FAKE, top=FAKE, status=FAKE, steady=3, mask=9, B=2, S=7, P=16, max_pages=8,
             stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_commit(a["alen"], a["toks"], a["nd"], a["ctx"], a["stride"], a["drafts"], a["out"],
                                      a["olen"], a["cap"], a["table"], a["used"], a["free"], a["top"], a["status"],
                                      a["steady"], a["mask"], a["B"], a["S"], a["P"], a["max_pages"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(alen=None), -1), (dict(status=None), -1), (dict(free=None), -1), (dict(drafts=None), -1),
    (dict(S=0), -2), (dict(S=65), -2), (dict(B=-1), -2), (dict(cap=-1), -2), (dict(steady=-1), -2), (dict(max_pages=0), -2),
    (dict(ctx=C.c_void_p(0x1002)), -4),
])
def test_commit_rejects_bad_arguments(kw, code):
    assert _commit(**kw) == code


def test_commit_empty_batch_is_ok_without_device():
    assert _commit(B=0) == 0


def _general(**kw):
    a = dict(logits=FAKE, drafts=FAKE, ql=None, qrow=None, qlse=None, seed=1, alen=FAKE, toks=FAKE, B=2, S=4, V=1024,
             ndu=1, nd=None, greedy=None, off=0, T=1.0, tau=0.0, samp=0, probs=None, dq=None, lse=None, ws=None,
             ws_bytes=0, stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_accept_general(a["logits"], a["drafts"], a["ql"], a["qrow"], a["qlse"], a["seed"],
                                              a["alen"], a["toks"], a["B"], a["S"], a["V"], a["ndu"], a["nd"],
                                              a["greedy"], a["off"], a["T"], a["tau"], a["samp"], a["probs"], a["dq"],
                                              a["lse"], a["ws"], a["ws_bytes"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(logits=None), -1), (dict(toks=None), -1), (dict(drafts=None), -1), (dict(ql=FAKE), -1),   # q_logits without q_row
    (dict(S=0), -2), (dict(V=1022), -2), (dict(ndu=4), -2), (dict(T=0.0), -2), (dict(T=-1.0), -2), (dict(tau=-0.5), -2),
    (dict(T=float("inf")), -2), (dict(T=float("nan")), -2),
    (dict(logits=ODD), -4), (dict(ql=ODD, qrow=FAKE), -4),
    (dict(), -5), (dict(ws=FAKE, ws_bytes=64), -5),
])
def test_general_accept_rejects_bad_arguments(kw, code):
    assert _general(**kw) == code


def test_general_accept_workspace_and_empty_batch():
    assert _general(B=0) == 0
    g = idlm.idlm_isd_accept_general_workspace(256, 16, 151936)
    assert g > idlm.idlm_isd_accept_workspace(256, 16, 151936) and g % 256 == 0
    assert idlm.idlm_isd_accept_general_workspace(4, 4, 1023) == 0


def _filtered(**kw):
    a = dict(logits=FAKE, drafts=FAKE, seed=1, alen=FAKE, toks=FAKE, B=2, S=4, V=1024, ndu=1, nd=None, greedy=None, off=0,
             T=1.0, tau=0.0, top_k=50, top_p=0.95, samp=0, probs=None, kept=None, ws=None, ws_bytes=0, stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_accept_filtered(a["logits"], a["drafts"], a["seed"], a["alen"], a["toks"], a["B"], a["S"],
                                               a["V"], a["ndu"], a["nd"], a["greedy"], a["off"], a["T"], a["tau"],
                                               a["top_k"], a["top_p"], a["samp"], a["probs"], a["kept"], a["ws"],
                                               a["ws_bytes"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(logits=None), -1), (dict(alen=None), -1), (dict(drafts=None), -1),
    (dict(S=65), -2), (dict(V=6), -2), (dict(top_k=0), -2), (dict(top_k=65), -2), (dict(top_p=0.0), -2), (dict(top_p=1.5), -2),
    (dict(T=0.0), -2), (dict(tau=-1.0), -2),
    (dict(logits=ODD), -4),
    (dict(), -5), (dict(ws=FAKE, ws_bytes=128), -5),
])
def test_filtered_accept_rejects_bad_arguments(kw, code):
    assert _filtered(**kw) == code


def test_filtered_accept_workspace_and_empty_batch():
    assert _filtered(B=0) == 0
    assert idlm.idlm_isd_accept_filtered_workspace(256, 16, 151936) == 256 * 16 * 64 * 8
    assert idlm.idlm_isd_accept_filtered_workspace(4, 4, 1023) == 0


def _filtered_q(**kw):
    a = dict(logits=FAKE, dtype=0, drafts=FAKE, q_cand=None, q_row=None, seed=1, alen=FAKE, toks=FAKE, B=2, S=4, V=1024, ndu=1, nd=None,
             greedy=None, off=0, T=1.0, tau=0.0, top_k=50, top_p=0.95, samp=0, probs=None, dq=None, kept=None, cand_out=None,
             ws=None, ws_bytes=0, stream=None)
    a.update(kw)
    return idlm.lib().idlm_isd_accept_filtered_q(a["logits"], a["dtype"], a["drafts"], a["q_cand"], a["q_row"], a["seed"], a["alen"],
                                                 a["toks"], a["B"], a["S"], a["V"], a["ndu"], a["nd"], a["greedy"], a["off"],
                                                 a["T"], a["tau"], a["top_k"], a["top_p"], a["samp"], a["probs"], a["dq"],
                                                 a["kept"], a["cand_out"], a["ws"], a["ws_bytes"], a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(logits=None), -1), (dict(q_cand=FAKE), -1),                       # proposer records without their row index
    (dict(top_k=65), -2), (dict(T=0.0), -2),
    (dict(dtype=2), -3), (dict(dtype=1, V=1028), -2), (dict(dtype=1, V=1032), -5),    # bf16 rows: whole 16-byte loads of 8 values
    (dict(q_cand=FAKE, q_row=FAKE, cand_out=FAKE), -2),                     # the proposer's record would be overwritten
    (dict(q_cand=ODD, q_row=FAKE), -4), (dict(cand_out=ODD), -4),
    (dict(), -5), (dict(q_cand=FAKE, q_row=FAKE), -5),                      # neither cand_out nor a workspace
])
def test_filtered_q_accept_rejects_bad_arguments(kw, code):
    assert _filtered_q(**kw) == code
    assert _filtered_q(B=0) == 0


def test_rng_dump_rejects_bad_arguments():
    f = idlm.lib().idlm_isd_rng_dump
    assert f(1, 0, 1, 0, 0, 64, None, None, None) == 0                 # no rows: nothing to do
    assert f(1, 0, 1, 0, 2, 64, None, None, None) == -1                # no output at all
    assert f(1, 0, 1, 0, 65536, 64, FAKE, None, None) == -2
    assert f(1, 0, 1, -1, 2, 64, FAKE, None, None) == -2 and f(1, 0, -1, 0, 2, 64, FAKE, None, None) == -2
    assert f(1, 0, 1, 0, 2, 0, FAKE, None, None) == -2
    assert f(1, 0, 1, 2**31 - 1, 2, 64, FAKE, None, None) == -2        # row numbers must stay below 2^31


def _lora(**kw):
    a = dict(x=FAKE, W=FAKE, A=FAKE, Bm=FAKE, gate=FAKE, nd=None, S=1, h=FAKE, T=32, d_in=256, d_out=512, r=128, tile=0,
             splits=0, ws=None, ws_bytes=0, stream=None)
    a.update(kw)
    return idlm.lib().idlm_gated_lora_linear(a["x"], a["W"], a["A"], a["Bm"], a["gate"], a["nd"], a["S"], a["h"], a["T"],
                                             a["d_in"], a["d_out"], a["r"], a["tile"], a["splits"], a["ws"], a["ws_bytes"],
                                             a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(x=None), -1), (dict(W=None), -1), (dict(h=None), -1), (dict(A=None), -1), (dict(Bm=None), -1),
    (dict(gate=None, nd=None), -1),
    (dict(d_in=96), -2), (dict(d_in=0), -2), (dict(d_out=12), -2), (dict(d_out=0), -2), (dict(r=32), -2), (dict(r=8192), -2),
    (dict(T=-1), -2), (dict(tile=32), -2), (dict(splits=17), -2), (dict(splits=-1), -2),
    (dict(gate=None, nd=FAKE, S=5), -2),            # T = 32 is not a whole number of strides of 5 rows
    (dict(gate=None, nd=FAKE, S=0), -2),
    (dict(x=ODD), -4), (dict(W=ODD), -4), (dict(h=ODD), -4), (dict(A=ODD), -4),
    (dict(), -5), (dict(ws=FAKE, ws_bytes=64), -5),
    (dict(T=0), 0),
])
def test_gated_lora_rejects_bad_arguments(kw, code):
    assert _lora(**kw) == code


def test_gated_lora_workspace_is_host_only():
    w = idlm.idlm_gated_lora_linear_workspace
    assert w(4096, 4096, 4096, 128, 0, 0) == 4096 * 128 * 2 + 4 * 4096 * 128 * 4     # u and the four partial sums of the shrink
    assert w(4096, 4096, 4096, 0, 256, 1) == 0                                       # plain base layer, one K part
    assert w(448, 4096, 4096, 128, 128, 4) >= 448 * 128 * 2 + 4 * 448 * 4096 * 4
    assert w(448, 4096, 4096, 128, 0, 0) % 256 == 0
    assert w(32, 96, 512, 128, 0, 0) == 0 and w(32, 256, 512, 128, 32, 0) == 0 and w(32, 256, 512, 128, 0, 17) == 0


def test_validate_checks_host_arguments_first():
    v = idlm.lib().idlm_isd_validate
    host = (C.c_int32 * 4)(9, 9, 9, 9)
    args = lambda **kw: [kw.get("table", FAKE), kw.get("ctx", FAKE), kw.get("S", 4), kw.get("B", 2), 16, 10, 4, FAKE, None, 1,
                         1024, kw.get("report", FAKE), host, None]
    assert v(*args(report=None)) == -1
    assert v(*args(S=0)) == -2 and v(*args(S=65)) == -2 and v(*args(B=-1)) == -2
    assert v(*args(B=0)) == 0 and list(host) == [0, -1, 0, 0]
