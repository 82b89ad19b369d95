"""GPU parity for eager emission (Sec. 3 taken literally; Sec. 4, Fig. 3): after every pushed
segment the announced activations of every layer equal the conventional network applied to the
input seen so far, the rest taken as zero.  Checked against the paper-literal eager oracle (tiny
nets, every layer after every row) and against the dense oracle on zero-extended inputs."""
import numpy as np
import pytest

import oracle
from oracle.eager import EagerNet
import workloads as wl_mod
from workloads import conv, maxpool
from helpers import TOL

pytestmark = pytest.mark.gpu


def _shapes(wl):
    shp = [(wl["in_h"], wl["in_w"], wl["in_c"])]
    for (h, w, c) in oracle.layer_shapes(wl["layers"], wl["in_h"], wl["in_w"]):
        shp.append((h, w, c))
    return shp


def _tiny(prec, seed, layers, H, W, C0, with_bias):
    rng = np.random.default_rng(seed)
    integer = prec == "i8"
    ws, bs = [], []
    for L in layers:
        if L["kind"] != "conv":
            ws.append(None); bs.append(None); continue
        shape = (L["c_out"], L["c_in"], L["k_h"], L["k_w"])
        if integer:
            ws.append(rng.integers(-4, 5, size=shape).astype(np.int8))
            bs.append(rng.integers(-6, 7, size=(L["c_out"],)).astype(np.int32) if with_bias else None)
        else:
            ws.append(rng.normal(0, 0.5, size=shape).astype(np.float32))
            bs.append(rng.normal(0, 0.3, size=(L["c_out"],)).astype(np.float32) if with_bias else None)
    x = rng.integers(0, 6, size=(2, H, W, C0)).astype(np.int8) if integer else rng.random((2, H, W, C0)).astype(np.float32)
    x[rng.random((2, H, W)) < 0.4] = 0
    return dict(name="tiny", precision=prec, in_h=H, in_w=W, in_c=C0, layers=layers, weights=ws, biases=bs, x=x,
                seg_rows=1, streams=2)


# which of the conv kernels serves the 3x3 / stride 1 / same-padded layers: the library's choice (register-tiled for float
# nets, event by event for quantised ones), or forced: tiled with eight positions per lane, tiled for a quantised net,
# event by event for a float net (the sizes of these tests pick two positions per lane by themselves)
KERNELS = [{}, {"IDF_EAGER_POS": "8"}, {"IDF_EAGER_TILED": "1"}, {"IDF_EAGER_TILED": "1", "IDF_EAGER_POS": "8"}, {"IDF_EAGER_POS": "4"},
           {"IDF_EAGER_TILED": "1", "IDF_EAGER_POS": "4"}, {"IDF_EAGER_PLAIN": "1"}]


@pytest.mark.parametrize("env", KERNELS, ids=lambda e: "+".join(f"{k[10:].lower()}{v}" for k, v in e.items()) or "default")
@pytest.mark.parametrize("prec,with_bias", [("f32", True), ("f32", False), ("i8", True), ("i8", False)])
def test_every_layer_after_every_row_against_the_literal_scheme(prec, with_bias, env, monkeypatch):
    import torch
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    q = dict(act="relu_shr_clamp", shr=2, clamp_hi=15) if prec == "i8" else {}
    layers = [conv(2, 4, 3, 3, p_h=1, p_w=1, **q), maxpool(4), conv(4, 3, 3, 3, p_h=1, p_w=1, **q),
              conv(3, 2, 3, 3, s=2, **({"act": "relu"} if prec == "i8" else {}))]
    wl = _tiny(prec, 3, layers, 10, 8, 2, with_bias)
    shp = _shapes(wl)
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 2)
    st.enable_eager()
    x = input_tensor(wl)
    dt = np.int64 if prec == "i8" else np.float64
    refs = [EagerNet(layers, 10, 8, 2, wl["weights"], wl["biases"], dtype=dt) for _ in range(2)]
    nb, kept = st.eager_state_bytes()
    whole = [shp[lv][0] for lv in range(len(layers) + 1)]
    if with_bias:
        assert kept.tolist() == whole                 # every neuron announces its bias before any input: all levels whole
    else:
        # the cone: the pushed row; the 3 rows it reaches in the first layer plus one the pool still looks at;
        # 2 pooled rows; the 4 rows those reach; the last level has 2 rows in all
        assert kept.tolist() == [1, 4, 2, 4, 2]
        assert nb < sum(4 * (2 if lv in (0, 2) else 3) * shp[lv][0] * shp[lv][1] * shp[lv][2] for lv in range(4))
    for r in range(10):
        st.push_segment(x[:, r:r + 1].contiguous())
        for b in range(2):
            refs[b].present_row(r, wl["x"][b, r])
        for lv in range(len(layers) + 1):
            got, first, cnt = st.read_announced_rows(lv, shp[lv][1:], shp[lv][0])
            got = got.cpu().numpy()
            for b in range(2):
                lo, n = int(first[b]), int(cnt[b])
                want = refs[b].announced[lv]
                assert n >= 1, (r, lv)
                if prec == "i8":
                    assert np.array_equal(got[b, :n].astype(np.int64), want[lo:lo + n]), (r, lv, b)
                else:
                    assert np.max(np.abs(got[b, :n] - want[lo:lo + n])) <= 1e-5 * max(1.0, np.max(np.abs(want))), (r, lv, b)
                if not with_bias:
                    assert not want[lo + n:].any(), (r, lv, b)      # rows not reached yet are all zero: nothing to keep
                elif lv == len(layers):
                    assert lo == 0 and n == shp[lv][0]
        # the output (last level) is also there as a whole map
        got = st.read_announced(len(layers), shp[-1]).cpu().numpy()
        for b in range(2):
            assert np.max(np.abs(got[b].astype(np.float64) - refs[b].announced[-1])) <= 1e-5 * max(1.0, np.max(np.abs(refs[b].announced[-1])))
    if not with_bias:
        with pytest.raises(idf.IdfError):
            st.read_announced(1, shp[1])                 # an inner level is a ring, not a map
    ev = st.get_stats(0)["events_in"]
    assert ev[0] == np.count_nonzero(wl["x"][0]) and (ev[1:] > 0).all()
    with pytest.raises(idf.IdfError):
        st.read_outputs(4)
    st.close(); net.destroy()


@pytest.mark.parametrize("cfg,kw,seg", [
    (3, dict(streams=3, size=16, channels=(8, 8, 16, 16)), 1),
    (3, dict(streams=2, size=16, channels=(8, 8, 16, 16)), 3),
    (4, dict(streams=2, size=24, channels=(4, 4, 8, 8, 16, 16, 16, 16)), 2),
    (5, dict(streams=2, size=24, channels=(8, 8, 16, 16, 16, 16, 16)), 1),
    (5, dict(streams=2, size=24, channels=(8, 8, 16, 16, 16, 16, 16)), 5),
])
@pytest.mark.parametrize("env", KERNELS[:6], ids=lambda e: "+".join(f"{k[10:].lower()}{v}" for k, v in e.items()) or "default")
def test_output_after_a_prefix_is_the_network_on_the_prefix(cfg, kw, seg, env, monkeypatch):
    import paper_1804_10727_amd as idf
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(cfg, **kw)
    shp = _shapes(wl)
    B, H = wl["streams"], wl["in_h"]
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, B, max_seg_rows=seg)
    st.enable_eager()
    x = input_tensor(wl)
    checks = {0, 2, H // seg // 2, (H + seg - 1) // seg - 1}
    for i, r in enumerate(range(0, H, seg)):
        st.push_segment(x[:, r:r + seg].contiguous())
        if i not in checks:
            continue
        got = st.read_announced(len(wl["layers"]), shp[-1]).cpu().numpy()
        for b in range(B):
            xp = wl["x"][b].copy()
            xp[r + seg:] = 0
            bf16 = wl["precision"] == "bf16"
            want = oracle.dense(wl["layers"], xp, wl["weights"], wl["biases"], integer=wl["precision"] == "i8",
                                emit_round="bf16" if bf16 else None)
            if wl["precision"] == "i8":
                assert np.array_equal(got[b].astype(np.int64), want), (i, b)
            else:
                tol = TOL["bf16_emul"] if bf16 else TOL["f32"]
                assert np.max(np.abs(got[b] - want)) <= tol * max(np.max(np.abs(want)), 1e-30), (i, b)
                if bf16:        # and within the wider bound of the net that rounds nothing
                    true = oracle.dense(wl["layers"], xp, wl["weights"], wl["biases"])
                    assert np.max(np.abs(got[b] - true)) <= TOL["bf16_true"] * max(np.max(np.abs(true)), 1e-30), (i, b)
    # second sample in the same streams: everything starts from zero again
    st.push_segment(x[:, 0:seg].contiguous())
    got = st.read_announced(len(wl["layers"]), shp[-1]).cpu().numpy()
    xp = wl["x"][0].copy(); xp[seg:] = 0
    want = oracle.dense(wl["layers"], xp, wl["weights"], wl["biases"], integer=wl["precision"] == "i8",
                        emit_round="bf16" if wl["precision"] == "bf16" else None)
    tol = TOL["bf16_emul"] if wl["precision"] == "bf16" else TOL["f32"]
    assert np.max(np.abs(got[0].astype(np.float64) - want)) <= tol * max(np.max(np.abs(want)), 1e-30)
    st.close(); net.destroy()
