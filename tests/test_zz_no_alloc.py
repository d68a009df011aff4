"""The entry point that allocates nothing (milora_layer_decode_noalloc), through the C ABI: two calls in a row on the
library's own scratch array, the second with a smaller input, each bit for bit what milora_layer_decode gives on a
caller's workspace (the same kernels in the same order), and within the parity tolerance of the oracle."""
import pytest
import torch

import oracle
from paper_2410_18035_amd import binding as mb
from paper_2410_18035_amd import synth
from tests.util import assert_rows_close, oracle_adapters

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(d, F, B, T, ranks, seed, rmsnorm, with_attn):
    wl = synth.Workload("noalloc", "bf16", d, F, 1, T, B, ranks, (4, 8), tenants="uniform", seed=seed, sigma_w=0.05,
                        sigma_lora=0.15)
    W = synth.base_weights(wl, 0, DEV)
    ad = synth.adapters(wl, 0, DEV)
    tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
    Wp = [mb.milora_pack_weight(w) for w in W]
    tid = synth.tenant_ids(wl)
    g = torch.Generator().manual_seed(seed)
    route = torch.randint(0, 7, (B,), generator=g).to(torch.uint8)
    route[0] = mb.ROUTE_SET | 0b1001001
    x = synth.decode_input(wl, 0, DEV)
    attn = synth.decode_input(wl, 1000, DEV) if with_attn else None
    # every buffer exists before the call under test
    y = torch.empty_like(x)
    qkv = torch.empty(B, 3 * d, dtype=x.dtype, device=DEV)
    tid_dev, route_dev = tid.to(DEV), route.to(DEV)
    y_ws, qkv_ws = mb.milora_layer_decode(x, Wp, tab, tid_dev, route_dev, F, w_layout=mb.W_PACKED, rmsnorm=rmsnorm,
                                          attn_out=attn)
    torch.cuda.synchronize()
    allocations = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]  # requests to torch's allocator so far
    before = allocations()
    mb.milora_layer_decode_noalloc(x, Wp, tab, tid_dev, route_dev, F, y, qkv_out=qkv, rmsnorm=rmsnorm, attn_out=attn)
    torch.cuda.synchronize()
    assert allocations() == before
    assert mb.milora_packed_workspace_status(None) == 0
    assert torch.equal(y, y_ws) and torch.equal(qkv, qkv_ws)
    y_ref, qkv_ref = oracle.layer_decode(synth.as_numpy(x), [synth.as_numpy(w) for w in W], oracle_adapters(ad), tid.numpy(),
                                         route.numpy(), F, flags=oracle.FLAG_RMSNORM if rmsnorm else 0,
                                         attn_out=None if attn is None else synth.as_numpy(attn))
    assert_rows_close(y, y_ref, torch.bfloat16, "y")
    assert_rows_close(qkv, qkv_ref, torch.bfloat16, "qkv")


def test_noalloc_layer_decode_two_calls_second_smaller():
    _case(d=1024, F=2752, B=32, T=6, ranks=(16, 32), seed=81, rmsnorm=True, with_attn=False)
    _case(d=512, F=1056, B=9, T=4, ranks=(8,), seed=82, rmsnorm=False, with_attn=True)


def test_noalloc_rejects_what_does_not_fit():
    wl = synth.Workload("noalloc", "bf16", 256, 352, 1, 2, 40, (8,), (4, 8), seed=83)
    W = synth.base_weights(wl, 0, DEV)
    ad = synth.adapters(wl, 0, DEV)
    tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
    Wp = [mb.milora_pack_weight(w) for w in W]
    x = synth.decode_input(wl, 0, DEV)
    tid = synth.tenant_ids(wl).to(DEV)
    route = torch.zeros(wl.B, dtype=torch.uint8, device=DEV)
    with pytest.raises(mb.MiloraError) as e:  # more than 32 rows
        mb.milora_layer_decode_noalloc(x, Wp, tab, tid, route, wl.F, torch.empty_like(x))
    assert e.value.status == -2
    with pytest.raises(mb.MiloraError) as e:  # fp32 has no packed layout
        mb.milora_layer_decode_noalloc(x[:8].float(), [w.float() for w in W], tab, tid[:8].contiguous(),
                                       route[:8].contiguous(), wl.F, torch.empty(8, wl.d, dtype=torch.float32, device=DEV))
    assert e.value.status == -3
