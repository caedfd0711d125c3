"""Full-sequence bidirectional attention (sdllm_dense_attn) against the oracle's plain attention."""
import numpy as np
import pytest
import torch

from oracle import sdllm_oracle as orc
from paper_2508_02558_amd import binding as B
from paper_2508_02558_amd import workloads as wl
from tests import parity_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _shape(Bt, Hq, Hkv, d, L, dtype, **kw):
    return B.make_shape(batch=Bt, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=L, block_off=0, block_len=min(32, L),
                        dtype=dtype, **kw)


@pytest.mark.parametrize("Bt,Hq,Hkv,L", [(1, 2, 2, 256), (2, 4, 2, 300), (1, 7, 1, 33), (3, 2, 2, 1), (1, 4, 4, 1000)])
def test_dense_attn_bf16_matches_oracle(Bt, Hq, Hkv, L):
    print(f"[case] dense_attn bf16 B={Bt} Hq={Hq} Hkv={Hkv} L={L}", flush=True)
    torch.manual_seed(L)
    d = 128
    q = torch.randn(Bt, Hq, L, d, device=DEV).bfloat16()
    k = torch.randn(Bt, Hkv, L, d, device=DEV).bfloat16()
    v = torch.randn(Bt, Hkv, L, d, device=DEV).bfloat16()
    out = torch.zeros(Bt, Hq, L, d, device=DEV, dtype=torch.bfloat16)
    B.sdllm_dense_attn(_shape(Bt, Hq, Hkv, d, L, B.SDLLM_BF16), q, k, v, out)
    torch.cuda.synchronize()
    U.assert_close(out, U.oracle_attention_batch(q, k, v), "bf16", f"L={L}")


@pytest.mark.parametrize("L", [31, 32, 64, 65, 96, 97, 128, 129, 191, 257])
def test_dense_attn_tile_and_stage_boundaries(L):
    # the kernel pipelines 32-key tiles through 64-key stages: every parity of tile and stage count,
    # with and without a ragged last tile
    print(f"[case] dense_attn boundaries L={L}", flush=True)
    torch.manual_seed(1000 + L)
    Bt, Hq, Hkv, d = 1, 2, 1, 128
    q = torch.randn(Bt, Hq, L, d, device=DEV).bfloat16()
    k = torch.randn(Bt, Hkv, L, d, device=DEV).bfloat16()
    v = torch.randn(Bt, Hkv, L, d, device=DEV).bfloat16()
    out = torch.zeros(Bt, Hq, L, d, device=DEV, dtype=torch.bfloat16)
    B.sdllm_dense_attn(_shape(Bt, Hq, Hkv, d, L, B.SDLLM_BF16), q, k, v, out)
    torch.cuda.synchronize()
    U.assert_close(out, U.oracle_attention_batch(q, k, v), "bf16", f"L={L}")


def test_dense_attn_generic_path_fp32_and_strided():
    print("[case] dense_attn fp32 / d=64 / strided", flush=True)
    torch.manual_seed(3)
    Bt, Hq, Hkv, L, d = 2, 4, 2, 90, 64
    q = torch.randn(Bt, Hq, L, d, device=DEV)
    k = torch.randn(Bt, Hkv, L, d, device=DEV)
    v = torch.randn(Bt, Hkv, L, d, device=DEV)
    out = torch.zeros_like(q)
    B.sdllm_dense_attn(_shape(Bt, Hq, Hkv, d, L, B.SDLLM_F32), q, k, v, out)
    torch.cuda.synchronize()
    U.assert_close(out, U.oracle_attention_batch(q, k, v), "f32", "fp32 d=64")
    # bf16, d=128, tensors stored [B, L, H, d] and passed as [B, H, L, d] views, explicit scale
    L, d = 200, 128
    q = torch.randn(Bt, L, Hq, d, device=DEV).bfloat16().permute(0, 2, 1, 3)
    k = torch.randn(Bt, L, Hkv, d, device=DEV).bfloat16().permute(0, 2, 1, 3)
    v = torch.randn(Bt, L, Hkv, d, device=DEV).bfloat16().permute(0, 2, 1, 3)
    out = torch.zeros(Bt, L, Hq, d, device=DEV, dtype=torch.bfloat16).permute(0, 2, 1, 3)
    B.sdllm_dense_attn(_shape(Bt, Hq, Hkv, d, L, B.SDLLM_BF16, softmax_scale=0.07, kv_stride=B.strides_of(k)), q, k, v, out)
    torch.cuda.synchronize()
    U.assert_close(out, U.oracle_attention_batch(q, k, v, scale=0.07), "bf16", "strided")


def test_dense_attn_block_rows_agree_with_block_step():
    # the block's rows of the full attention are what sdllm_block_step returns at cache_state 0
    print("[case] dense_attn vs block_step", flush=True)
    w = wl.WORKLOADS["llada8b_layer"].scaled(n_q_heads=4, n_kv_heads=4, prompt=512, gen=128)
    inp = wl.make_block_inputs(w, n_steps=1, device=DEV)
    o, b = inp["block_off"], w.block
    shape = U.shape_for(w)
    gl = U.GpuLayer(shape, DEV)
    k, v = inp["k_full"], inp["v_full"]
    q_full = torch.randn(w.batch, w.n_q_heads, w.seq_len, w.head_dim, device=DEV).bfloat16()
    q_full[:, :, o:o + b] = inp["q"][0]
    out_full = torch.zeros_like(q_full)
    B.sdllm_dense_attn(shape, q_full, k, v, out_full)
    gl.block_step(0, 1, inp["q"][0].contiguous(), k, v)
    torch.cuda.synchronize()
    assert (out_full[:, :, o:o + b].float() - gl.out.float()).abs().max().item() <= 1.6e-2   # two bf16 roundings
    U.assert_close(out_full, U.oracle_attention_batch(q_full, k, v), "bf16", "full rows")


def test_dense_attn_full_size_sampled_rows():
    # LLaDA-8B-shaped layer at the 4k-prompt length, one batch element; sampled heads against the oracle
    print("[case] dense_attn full size", flush=True)
    torch.manual_seed(11)
    Bt, H, L, d = 1, 32, 4352, 128
    q = torch.randn(Bt, H, L, d, device=DEV).bfloat16()
    k = torch.randn(Bt, H, L, d, device=DEV).bfloat16()
    v = torch.randn(Bt, H, L, d, device=DEV).bfloat16()
    out = torch.zeros_like(q)
    B.sdllm_dense_attn(_shape(Bt, H, H, d, L, B.SDLLM_BF16), q, k, v, out)
    torch.cuda.synchronize()
    for h in (0, 13, 31):
        ref = orc.attention(wl.to_f64(q[0, h:h + 1]), wl.to_f64(k[0, h:h + 1]), wl.to_f64(v[0, h:h + 1]))
        U.assert_close(out[0, h:h + 1], ref, "bf16", f"head {h}")
    assert torch.isfinite(out.float()).all()


def test_dense_attn_peaked_softmax():
    # logits spread over several dozen, and for every query row a dominant key late in the sequence
    print("[case] dense_attn peaked softmax", flush=True)
    torch.manual_seed(21)
    Bt, Hq, Hkv, L, d = 1, 4, 2, 520, 128
    q = (4.0 * torch.randn(Bt, Hq, L, d, device=DEV)).bfloat16()
    k = (4.0 * torch.randn(Bt, Hkv, L, d, device=DEV)).bfloat16()
    v = torch.randn(Bt, Hkv, L, d, device=DEV).bfloat16()
    k[:, :, 400] = (1.5 * q[:, ::2, 7].float()).bfloat16()
    out = torch.zeros(Bt, Hq, L, d, device=DEV, dtype=torch.bfloat16)
    B.sdllm_dense_attn(_shape(Bt, Hq, Hkv, d, L, B.SDLLM_BF16), q, k, v, out)
    torch.cuda.synchronize()
    U.assert_close(out, U.oracle_attention_batch(q, k, v), "bf16", "peaked")
