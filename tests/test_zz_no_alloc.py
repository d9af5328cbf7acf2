"""The decode span-attention entry point that allocates nothing (its partial records live in a
device array of the library) against the entry point that takes a caller workspace: two calls in a
row, the second on a smaller input, so that the second call finds the first call's records in the
shared array; then the same pair in the opposite order of sizes, and the size limit."""
import pytest
import torch

from paper_2601_18401_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(seed, Hq, Hkv, L, D, S, k, dtype):
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn((Hq, 1, D), generator=g).to(dtype).to(DEV)
    K = torch.randn((Hkv, L, D), generator=g).to(dtype).to(DEV)
    V = torch.randn((Hkv, L, D), generator=g).to(dtype).to(DEV)
    idx = B.sl_span_search_decode(Q, K, None, S, k)
    return Q, K, V, idx


def _compare(Q, K, V, idx, S, dtype):
    O_ref, LSE_ref = B.sl_span_attention_decode(Q, K, V, idx, S)
    out = (torch.full_like(O_ref, float("nan")), torch.full_like(LSE_ref, float("nan")))
    B.sl_span_attention_decode_noalloc(Q, K, V, idx, S, out)
    torch.cuda.synchronize()
    tol = 2e-2 if dtype == torch.bfloat16 else 1e-4
    assert float((out[0].float() - O_ref.float()).abs().max()) <= tol
    assert float((out[1] - LSE_ref).abs().max()) <= tol
    # same kernels on the same inputs: in fact bit-equal
    assert torch.equal(out[0], O_ref) and torch.equal(out[1], LSE_ref)


def test_noalloc_decode_matches_workspace_entry_point_on_two_calls_in_a_row():
    big = _case(1, 32, 4, 262144, 128, 512, 16, torch.bfloat16)      # 1.1 MB of partial records
    small = _case(2, 8, 2, 5000, 128, 96, 6, torch.bfloat16)         # ragged, far fewer records
    _compare(*big, 512, torch.bfloat16)
    _compare(*small, 96, torch.bfloat16)
    tiny = _case(3, 4, 4, 40, 64, 64, 4, torch.float32)              # no candidate span at all, fp32, D = 64
    _compare(*tiny, 64, torch.float32)
    _compare(*big, 512, torch.bfloat16)


def test_noalloc_decode_rejects_what_does_not_fit_its_array():
    assert B.sl_noalloc_scratch_bytes() == 8 << 20
    Hq, Hkv, D, S, k = 32, 4, 128, 16384, 32          # 33 slots x 32 chunks x 32 heads x 520 B = 17.6 MB
    L = 2 * S
    g = torch.Generator().manual_seed(4)
    Q = torch.randn((Hq, 1, D), generator=g).to(torch.bfloat16).to(DEV)
    K = torch.randn((Hkv, L, D), generator=g).to(torch.bfloat16).to(DEV)
    idx = torch.full((Hq, 1, k), -1, dtype=torch.int32, device=DEV)
    out = (torch.zeros((Hq, 1, D), dtype=torch.bfloat16, device=DEV), torch.zeros((Hq, 1), device=DEV))
    with pytest.raises(B.SlError) as e:
        B.sl_span_attention_decode_noalloc(Q, K, K, idx, S, out)
    assert e.value.status == 2
