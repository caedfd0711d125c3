"""sdllm_sparse_attn_noalloc (the entry point for callers that cannot allocate: its split-KV partials live
in a static device array inside the library) against sdllm_sparse_attn with a caller workspace, through
the C ABI: two calls in a row on the same GPU, the second with a smaller input, both with key splits so
that the scratch array is really used."""
import pytest
import torch

from paper_2508_02558_amd import binding as B
from tests import parity_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(Bt, Hq, Hkv, n_cached, seed):
    b, d = 32, 128
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    rn = lambda *shape: torch.randn(*shape, device=DEV, generator=g).bfloat16()
    shape = B.make_shape(batch=Bt, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=8192, block_off=4096,
                         block_len=b, dtype=B.SDLLM_BF16, cache_rows=n_cached)
    return shape, rn(Bt, Hq, b, d), rn(Bt, Hkv, n_cached, d), rn(Bt, Hkv, n_cached, d), rn(Bt, Hkv, b, d), rn(Bt, Hkv, b, d)


def test_noalloc_entry_matches_the_workspace_entry_on_two_calls_in_a_row():
    # 8 heads x 2000 cached keys -> 5 key splits; then 8 heads x 700 keys -> 2 key splits (fewer, shorter
    # partials in the same array, which still holds the first call's)
    for n_cached, seed in ((2000, 11), (700, 12)):
        print(f"[case] noalloc n_cached={n_cached}", flush=True)
        shape, q, kc, vc, kb, vb = _case(1, 8, 8, n_cached, seed)
        need = B.sdllm_workspace_bytes(shape, B.SDLLM_OP_SPARSE_ATTN, n_cached)
        assert 32 * 128 * 4 * 8 * 2 <= need <= B.SDLLM_STATIC_SCRATCH_BYTES   # at least two splits per head
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        want = torch.zeros_like(q)
        B.sdllm_sparse_attn(shape, q, kc, vc, n_cached, kb, vb, want, ws)
        got = torch.full_like(q, float("nan"))
        B.sdllm_sparse_attn_noalloc(shape, q, kc, vc, n_cached, kb, vb, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"n_cached={n_cached}: differs from sdllm_sparse_attn"
        ref = U.oracle_attention_batch(q, torch.cat([kc, kb], 2), torch.cat([vc, vb], 2))
        U.assert_close(got, ref, "bf16", f"noalloc n_cached={n_cached}")
