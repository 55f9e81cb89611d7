"""CPU-side tests of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad arguments before touching the GPU, and its host logic (rate rounding, weight
repacking, the CC workers) agrees with the oracle.  No GPU compute is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2411_15715_amd as si
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    hdr = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(si_[a-z_0-9]+)\s*\(", hdr))
    assert {"si_layer_create", "si_layer_forward", "si_route", "si_layer_destroy", "si_last_error"} <= declared
    L = si.lib()
    for name in declared:
        assert hasattr(L, name), "missing export " + name
    assert declared == set(si.EXPORTS)
    assert "gfx950" in si.si_version()


def test_split_counts_match_golden_and_oracle(oracle):
    rows = [ln.split() for ln in open(os.path.join(ROOT, "tests", "golden", "split_counts.txt")) if ln.strip() and ln[0] != "#"]
    for H, g, rgg, rcg, rcc, ngg, ncg, ncc in rows:
        assert si.si_split_counts(int(H), int(g), float(rgg), float(rcg)) == (int(ngg), int(ncg), int(ncc))
    for H, g in [(704, 64), (6400, 128), (28672, 64)]:
        for i in range(0, 11):
            for j in range(0, 11 - i):
                n_cc, n_cg, n_gg = oracle.split_counts(H, g, i / 10, j / 10)
                assert si.si_split_counts(H, g, i / 10, j / 10) == (n_gg, n_cg, n_cc)
    with pytest.raises(si.ScheInferError) as ei:
        si.si_split_counts(700, 64, 0.5, 0.5)
    assert ei.value.code == si.SI_EINVAL


def _desc(**kw):
    d = dict(d_model=256, d_ff=704, n_experts=1, top_k=1, d_ff_shared=0, r_gg=0.4, r_cg=0.3, r_cc=0.3, granule=0,
             max_tokens=32, cc_threads=0, device=0, stage_mib=0, n_stage=0)
    d.update(kw)
    return si.si_layer_desc_t(**d)


def test_create_rejects_bad_arguments_before_any_gpu_call():
    L = si.lib()
    w = np.zeros(704 * 256, np.uint16)
    p = ctypes.c_void_p(w.ctypes.data)
    out = ctypes.c_void_p(None)
    bad = [dict(d_model=250), dict(d_ff=700), dict(top_k=2), dict(n_experts=0), dict(r_gg=0.8), dict(r_cc=-0.1, r_gg=0.8),
           dict(granule=48), dict(max_tokens=0), dict(d_ff_shared=100), dict(n_stage=1), dict(n_experts=300, top_k=2)]
    for kw in bad:
        d = _desc(**kw)
        assert L.si_layer_create(ctypes.byref(d), p, p, p, None, None, None, ctypes.byref(out)) == si.SI_EINVAL, kw
        assert si.si_last_error() != ""
        assert out.value is None
    d = _desc()
    assert L.si_layer_create(ctypes.byref(d), None, p, p, None, None, None, ctypes.byref(out)) == si.SI_EINVAL
    d = _desc(d_ff_shared=128)
    assert L.si_layer_create(ctypes.byref(d), p, p, p, None, None, None, ctypes.byref(out)) == si.SI_EINVAL
    assert L.si_layer_create(None, p, p, p, None, None, None, ctypes.byref(out)) == si.SI_EINVAL
    assert L.si_layer_forward(None, None, None, 1, 0, 0, None, None, None) == si.SI_EINVAL
    assert L.si_layer_split_info(None, None, None, None, None, None, None) == si.SI_EINVAL
    assert L.si_layer_stats(None, None) == si.SI_EINVAL
    assert L.si_route(None, 1, 4, 2, None, None) == si.SI_EINVAL
    L.si_layer_destroy(None)  # allowed


def test_create_without_gpu_reports_hip_error():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    L = si.lib()
    w = np.zeros(704 * 256, np.uint16)
    p = ctypes.c_void_p(w.ctypes.data)
    out = ctypes.c_void_p(None)
    d = _desc()
    assert L.si_layer_create(ctypes.byref(d), p, p, p, None, None, None, ctypes.byref(out)) == si.SI_EHIP
    assert "device" in si.si_last_error().lower()


def _panel_width(M):
    p = 512
    while M % p:
        p //= 2
    return p


def _ntile_width(M):
    p = 256
    while M % p:
        p //= 2
    return p


@pytest.mark.parametrize("M", [64, 192, 1024])
def test_repack_layout(M):
    """gate / up block: [M/PW panels][64 j][PW m]; down block: [M/NW tiles][8 q][NW m][8 i] = Wd[j0+8q+i][m]."""
    rng = np.random.default_rng(1)
    H = 192
    PW, NW = _panel_width(M), _ntile_width(M)
    wg, wu, wd = (rng.integers(0, 65535, (H, M), dtype=np.uint16) for _ in range(3))
    out = si.si_repack_chunks(wg, wu, wd, 1, 2).reshape(2, 3 * 64 * M)
    for ci, c in enumerate((1, 2)):
        blk = out[ci]
        for f, src in enumerate((wg, wu)):
            panels = blk[f * 64 * M:(f + 1) * 64 * M].reshape(M // PW, 64, PW)
            ref = src[c * 64:(c + 1) * 64].reshape(64, M // PW, PW).transpose(1, 0, 2)
            assert np.array_equal(panels, ref)
        down = blk[128 * M:].reshape(M // NW, 8, NW, 8)  # [tile][q][m][i]
        ref = wd[c * 64:(c + 1) * 64].reshape(8, 8, M // NW, NW).transpose(2, 0, 3, 1)
        assert np.array_equal(down, ref)
    with pytest.raises(si.ScheInferError):
        si.si_repack_chunks(wg, wu, wd, 2, 2)


def _pack_host(w, key_g, key_u, key_d, n_chunks):
    E = w[key_g].shape[0] if w[key_g].ndim == 3 else 1
    g, u, d = (w[k].reshape(E, -1, w[k].shape[-1]) for k in (key_g, key_u, key_d))
    return np.concatenate([si.si_repack_chunks(g[e], u[e], d[e], 0, n_chunks) for e in range(E)])


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("T1,threads", [(1, 3), (5, 4), (40, 4)])
def test_cc_workers_match_oracle_cc_partial(oracle, T1, threads, generic, monkeypatch):
    """The CC partial (columns [0, n_cc) of every expert, Eq. 2) from the host workers equals the
    oracle evaluated on those columns alone.  Both code paths of the workers: the AVX-512 BF16 one (taken where
    the CPU has it) and the portable one."""
    if generic:
        monkeypatch.setenv("SI_CC_GENERIC", "1")
    else:
        monkeypatch.delenv("SI_CC_GENERIC", raising=False)
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128, d_ff=256, d_ff_shared=384, n_experts=8, top_k=3)
    w = synth.make_weights(cfg)
    xb = synth.make_tokens(cfg, T1)
    lg = synth.make_router_logits(cfg, xb)
    r = oracle.route(lg, cfg.top_k)
    n_cc, s_cc = 128, 192
    routed = _pack_host(w, "w_gate", "w_up", "w_down", n_cc // 64 + 1)  # one extra chunk (CG) behind the CC range
    shared = _pack_host(w, "s_gate", "s_up", "s_down", s_cc // 64)
    stride = (n_cc // 64 + 1) * 3 * 64 * cfg.d_model
    ycc = si.si_cc_compute(xb, r["idx"], r["w"].astype(np.float32), cfg.n_experts, routed, stride, n_cc // 64,
                           shared=shared, s_cc_chunks=s_cc // 64, threads=threads)
    ref = oracle.layer_forward(xb, w["w_gate"][:, :n_cc], w["w_up"][:, :n_cc], w["w_down"][:, :n_cc], logits=lg,
                               top_k=cfg.top_k, shared=tuple(w[k][:s_cc] for k in ("s_gate", "s_up", "s_down")))
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(ycc - ref)) <= 1e-4 * rms  # fp32 accumulation on exact bf16 inputs
    # dense, no shared expert
    d = synth.scaled(synth.CONFIGS["tiny_dense"], d_model=128, d_ff=256)
    wd_ = synth.make_weights(d)
    xd = synth.make_tokens(d, T1)
    packed = _pack_host(wd_, "w_gate", "w_up", "w_down", 3)
    y2 = si.si_cc_compute(xd, np.zeros((T1, 1), np.int32), np.ones((T1, 1), np.float32), 1, packed, 0, 3, threads=threads)
    ref2 = oracle.layer_forward(xd, wd_["w_gate"][:, :192], wd_["w_up"][:, :192], wd_["w_down"][:, :192])
    assert np.max(np.abs(y2 - ref2)) <= 1e-4 * np.sqrt(np.mean(ref2 ** 2))


# ------------------------------------------------------------------ 4-bit storage form
def _codes(q):
    """[.., M/2] bytes -> [.., M] codes (element m: low nibble of byte m/2 for even m)."""
    return np.stack([q & 15, q >> 4], axis=-1).reshape(q.shape[:-1] + (q.shape[-1] * 2,)).astype(np.uint32)


@pytest.mark.parametrize("M", [64, 192, 1024])
def test_repack_layout_q4(M):
    """Per chunk, bytes: gate codes | up codes | down codes | gate scales | up scales | down scales (32M each for the
    codes, 2M each for the scales); nibble orders as the kernels expect them."""
    rng = np.random.default_rng(2)
    H, NW = 192, _ntile_width(M)
    wq = {k: rng.integers(0, 256, (H, M // 2), dtype=np.uint8) for k in ("q_gate", "q_up", "q_down")}
    wq.update({k: rng.integers(0, 65535, (H, M // 64), dtype=np.uint16) for k in ("z_gate", "z_up")})
    wq["z_down"] = rng.integers(0, 65535, (H // 64, M), dtype=np.uint16)
    out = si.si_repack_chunks_q4(wq, 1, 2).reshape(2, 51 * M)
    for ci, c in enumerate((1, 2)):
        raw = out[ci].view(np.uint8)
        assert raw.size == 102 * M
        for f, (qk, zk) in enumerate((("q_gate", "z_gate"), ("q_up", "z_up"))):
            words = raw[32 * M * f:32 * M * (f + 1)].view(np.uint32).reshape(64, M // 8)
            codes = _codes(wq[qk][c * 64:(c + 1) * 64]).reshape(64, M // 8, 8)
            ref = np.zeros((64, M // 8), np.uint32)
            for e in range(8):
                ref |= codes[:, :, e] << np.uint32(4 * ((e >> 1) + 4 * (e & 1)))
            assert np.array_equal(words, ref)
            scales = raw[96 * M + 2 * M * f:96 * M + 2 * M * (f + 1)].view(np.uint16).reshape(64, M // 64)
            assert np.array_equal(scales, wq[zk][c * 64:(c + 1) * 64])
        words = raw[64 * M:96 * M].view(np.uint32).reshape(M // NW, 2, NW, 4)       # [tile][half][m][word]
        codes = _codes(wq["q_down"][c * 64:(c + 1) * 64])                             # [64 j][M]
        cj = codes.reshape(2, 4, 8, M // NW, NW)                                      # [half][word][e][tile][m]
        ref = np.zeros((M // NW, 2, NW, 4), np.uint32)
        for e in range(8):
            nib = 2 * e if e < 4 else 2 * (e - 4) + 1
            ref |= cj[:, :, e].transpose(2, 0, 3, 1) << np.uint32(4 * nib)
        assert np.array_equal(words, ref)
        assert np.array_equal(raw[100 * M:].view(np.uint16), wq["z_down"][c])
    with pytest.raises(si.ScheInferError):
        si.si_repack_chunks_q4(wq, 2, 2)


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("T1,threads", [(1, 3), (6, 4), (40, 4)])
def test_cc_workers_q4_match_oracle_cc_partial(oracle, T1, threads, generic, monkeypatch):
    if generic:
        monkeypatch.setenv("SI_CC_GENERIC", "1")
    else:
        monkeypatch.delenv("SI_CC_GENERIC", raising=False)
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128, d_ff=256, d_ff_shared=384, n_experts=8, top_k=3)
    wq = synth.make_weights_q4(cfg)
    xb = synth.make_tokens(cfg, T1)
    lg = synth.make_router_logits(cfg, xb)
    r = oracle.route(lg, cfg.top_k)
    n_cc, s_cc = 128, 192
    nch = n_cc // 64 + 1                  # one extra chunk (CG) behind the CC range
    routed = np.concatenate([si.si_repack_chunks_q4({k: wq[k][e] for k in ("q_gate", "q_up", "q_down", "z_gate", "z_up", "z_down")}, 0, nch)
                             for e in range(cfg.n_experts)])
    shared = si.si_repack_chunks_q4(wq, 0, s_cc // 64, prefix="s")
    ycc = si.si_cc_compute(xb, r["idx"], r["w"].astype(np.float32), cfg.n_experts, routed, nch * 51 * cfg.d_model, n_cc // 64,
                           shared=shared, s_cc_chunks=s_cc // 64, threads=threads, q4=True)
    cut = {k: (v[:, :n_cc] if k.startswith(("q_", "z_g", "z_u")) else v) for k, v in wq.items() if not k.startswith("s")}
    cut["z_down"] = wq["z_down"][:, :n_cc // 64]
    for k in ("sq_gate", "sq_up", "sq_down", "sz_gate", "sz_up"):
        cut[k] = wq[k][:s_cc]
    cut["sz_down"] = wq["sz_down"][:s_cc // 64]
    ref = oracle.layer_forward_q4(xb, cut, logits=lg, top_k=cfg.top_k)
    assert np.max(np.abs(ycc - ref)) <= 1e-4 * np.sqrt(np.mean(ref ** 2))
