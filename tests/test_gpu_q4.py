"""GPU parity of the 4-bit storage form: the HIP path (decode GEMVs straight from the codes, prompt-phase GEMMs
on bf16 copies made on the GPU, host workers on the codes) against the oracle, which dequantises exactly in
double.  Same bar as the bf16 layer: max-abs error <= 2e-2 x RMS."""
import numpy as np
import pytest
import torch

import paper_2411_15715_amd as si
import synth
from gpu_helpers import assert_parity

pytestmark = pytest.mark.gpu


class Q4Layer:
    def __init__(self, cfg, wq, split, max_tokens, **kw):
        self.cfg = cfg
        self.h = si.si_layer_create_q4(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k, wq, split[0], split[1], split[2],
                                       max_tokens, d_ff_shared=cfg.d_ff_shared, **kw)
        self.info = si.si_layer_split_info(self.h)

    def forward(self, x_bits, logits, n_g=0, mode=si.SI_AUTO):
        dev = torch.device("cuda:0")
        T = x_bits.shape[0]
        x = torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).to(dev)
        lg = torch.from_numpy(logits).to(dev) if logits is not None else None
        y = torch.full((T, self.cfg.d_model), float("nan"), dtype=torch.float32, device=dev)
        si.si_layer_forward(self.h, x.data_ptr(), lg.data_ptr() if lg is not None else None, T, n_g, mode, y.data_ptr(),
                            stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return y.cpu().numpy()

    def close(self):
        si.si_layer_destroy(self.h)


SPLITS = [(1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (0.0, 0.0, 1.0), (0.4, 0.3, 0.3), (0.2, 0.6, 0.2)]


@pytest.mark.parametrize("split", SPLITS)
def test_dense_q4(oracle, split):
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=512, d_ff=1792)
    wq = synth.make_weights_q4(cfg)
    L = Q4Layer(cfg, wq, split, max_tokens=300, stage_mib=1)
    try:
        for T, stream in ((1, 2), (6, 3)):
            xb = synth.make_tokens(cfg, T, stream=stream)
            assert_parity(L.forward(xb, None), oracle.layer_forward_q4(xb, wq))
        x16 = synth.make_tokens(cfg, 16, stream=4)
        assert_parity(L.forward(x16, None, n_g=5, mode=si.SI_DECODE), oracle.layer_forward_q4(x16, wq))
        xp = synth.make_tokens(cfg, 300)
        yo = oracle.layer_forward_q4(xp, wq)
        for n_g in (0, 100, 300):
            assert_parity(L.forward(xp, None, n_g=n_g), yo)
    finally:
        L.close()


@pytest.mark.parametrize("split", SPLITS)
def test_moe_q4(oracle, split):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=512, d_ff=1024)
    wq = synth.make_weights_q4(cfg)
    L = Q4Layer(cfg, wq, split, max_tokens=700, stage_mib=1)
    try:
        for T, stream in ((1, 1), (3, 2), (8, 3)):
            xb = synth.make_tokens(cfg, T, stream=stream)
            lg = synth.make_router_logits(cfg, xb)
            assert_parity(L.forward(xb, lg), oracle.layer_forward_q4(xb, wq, logits=lg, top_k=cfg.top_k))
        xp = synth.make_tokens(cfg, 700)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle.layer_forward_q4(xp, wq, logits=lg, top_k=cfg.top_k)
        for n_g in (0, 333, 700):
            assert_parity(L.forward(xp, lg, n_g=n_g), yo)
    finally:
        L.close()


@pytest.mark.parametrize("split", [(1.0, 0.0, 0.0), (0.4, 0.3, 0.3)])
def test_shared_expert_and_odd_width_q4(oracle, split):
    # Qwen-shaped: many experts, top-8, shared expert, Zipf routing; d_model = 192 is not a multiple of 128
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=192, d_ff=384, d_ff_shared=1024, n_experts=32)
    wq = synth.make_weights_q4(cfg)
    L = Q4Layer(cfg, wq, split, max_tokens=600, stage_mib=1)
    try:
        xd = synth.make_tokens(cfg, 4, stream=1)
        lg = synth.make_router_logits(cfg, xd)
        assert_parity(L.forward(xd, lg), oracle.layer_forward_q4(xd, wq, logits=lg, top_k=cfg.top_k))
        xp = synth.make_tokens(cfg, 600)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle.layer_forward_q4(xp, wq, logits=lg, top_k=cfg.top_k)
        for n_g in (0, 250):
            assert_parity(L.forward(xp, lg, n_g=n_g), yo)
    finally:
        L.close()


@pytest.mark.parametrize("split", [(1.0, 0.0, 0.0), (0.4, 0.3, 0.3)])
def test_two_pass_prompt_phase_q4(oracle, split):
    """deq_mib > 0: the prompt phase goes through a dequantisation kernel and the bf16 GEMMs instead of the GEMMs
    that read the codes; a 1 MiB scratch forces several sub-pieces per part.  Same bar, and close to the default."""
    for name, kw in (("llama2_70b", dict(d_model=512, d_ff=1792)), ("mixtral_8x7b", dict(d_model=512, d_ff=1024))):
        cfg = synth.scaled(synth.CONFIGS[name], **kw)
        wq = synth.make_weights_q4(cfg)
        xp = synth.make_tokens(cfg, 300)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle.layer_forward_q4(xp, wq, logits=lg, top_k=cfg.top_k)
        outs = []
        for deq_mib in (1, 0):
            L = Q4Layer(cfg, wq, split, max_tokens=300, stage_mib=1, deq_mib=deq_mib)
            try:
                for n_g in (0, 120):
                    y = L.forward(xp, lg, n_g=n_g)
                    assert_parity(y, yo)
                outs.append(y)
            finally:
                L.close()
        # both paths multiply by the same bf16((code - 8) * scale): they differ only in the order of fp32 sums
        rms = float(np.sqrt(np.mean(yo ** 2)))
        assert np.max(np.abs(outs[0] - outs[1])) <= 1e-3 * rms


def test_full_size_mixtral_q4(oracle):
    """Mixtral-8x7B-shaped layer at full size, 50/50/0: decode on all tokens, prefill on sampled tokens."""
    cfg = synth.CONFIGS["mixtral_8x7b"]
    wq = synth.make_weights_q4(cfg, threads=16)
    L = Q4Layer(cfg, wq, cfg.split, max_tokens=cfg.t_prefill)
    try:
        xd = synth.make_tokens(cfg, 2, stream=1)
        lg = synth.make_router_logits(cfg, xd)
        assert_parity(L.forward(xd, lg), oracle.layer_forward_q4(xd, wq, logits=lg, top_k=cfg.top_k))
        xp = synth.make_tokens(cfg, cfg.t_prefill)
        lg = synth.make_router_logits(cfg, xp)
        sel = np.linspace(0, cfg.t_prefill - 1, 12).astype(np.int32)
        yo = oracle.layer_forward_q4(xp, wq, logits=lg, top_k=cfg.top_k, sel=sel)
        assert_parity(L.forward(xp, lg)[sel], yo)
    finally:
        L.close()
