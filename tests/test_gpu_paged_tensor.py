"""PagedTensor on the device's virtual memory management (Sec. 4.1): stable per-layer addresses
over two reusable physical blocks, dedicated blocks for uncompressed-resident layers, and a
kernel that knows nothing about paging consuming the weights through those addresses."""
import numpy as np
import pytest
import torch

from oracle import ffn as offn
from oracle import paging as opg
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import harness, inputs

pytestmark = pytest.mark.gpu


def read_u16(addr, n_elems):
    """Copy n_elems 16-bit words from a raw device address with the library's plain copy kernel."""
    out = torch.empty(n_elems, dtype=torch.int16, device="cuda")
    B.fluxmoe_stream_copy(out.data_ptr(), addr, n_elems * 2, 64)
    torch.cuda.synchronize()
    return out


def write_u16(addr, t):
    B.fluxmoe_stream_copy(addr, t.data_ptr(), t.numel() * 2, 64)
    torch.cuda.synchronize()


def test_layers_alias_two_reusable_blocks_and_feed_an_unaware_kernel():
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_layers=4, n_experts=8, n_slots=16)
    N, L, H, F = cfg.n_layers, cfg.n_experts, cfg.hidden, cfg.ffn
    pt = B.fluxmoe_paged_tensor_create(N, L, H, F)
    ctx = B.fluxmoe_create(N, L, H, F, 2 * L)
    keep = []
    try:
        info = B.fluxmoe_paged_tensor_info_get(pt)
        lay = opg.paged_tensor_layout(N, L, H, F, info.granularity)
        assert info.pad_bytes == lay["M_pad"] == 0
        assert info.physical_bytes == 2 * (lay["S"][1] + lay["S"][2])
        for d in (1, 2):
            assert info.v0[d - 1] % info.granularity == 0
            for i in (0, 3):
                for e in (0, L - 1):
                    assert B.fluxmoe_paged_tensor_address(pt, i, d, e) == opg.paged_tensor_address(
                        info.v0[d - 1], lay["S"][d], lay["sigma"][d], i + 1, e + 1)
        # the context's slot arenas are the reusable window: slots [0, L) = F_0, [L, 2L) = F_1
        sizes = B.fluxmoe_query_sizes(ctx)
        ws_bytes = int(sizes.pool_workspace_bytes + B.fluxmoe_ffn_workspace_bytes(ctx, cfg.tokens, cfg.top_k, True))
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
        page_table = torch.full((N, L), -1, dtype=torch.int32, device="cuda")
        B.fluxmoe_bind_arenas(ctx, info.reusable_window[0], info.reusable_window[1], ws.data_ptr(), ws_bytes)
        dense = {}
        for layer in range(N):
            w13, w2 = harness.make_layer_on_host(cfg, layer)
            blob = torch.empty(int(sizes.layer_blob_bound), dtype=torch.uint8)
            used = B.fluxmoe_encode_pool(ctx, layer, w13.data_ptr(), w2.data_ptr(), blob.data_ptr(), blob.numel())
            dev = blob[:used].cuda()
            keep.append(dev)
            B.fluxmoe_bind_layer(ctx, layer, dev.data_ptr())
            dense[layer] = (w13, w2)
        B.fluxmoe_reset_page_table(ctx, page_table.data_ptr())
        ids = np.arange(L, dtype=np.int32)

        def materialize(layer):
            B.fluxmoe_materialize(ctx, layer, ids, page_table.data_ptr(), (layer & 1) * L + ids)
            torch.cuda.synchronize()
            assert B.fluxmoe_device_errors(ctx) == 0

        def layer_shows(at_layer, weights_of):
            for e in (0, 3, L - 1):
                a = read_u16(B.fluxmoe_paged_tensor_address(pt, at_layer, 1, e), 2 * H * F)
                b = read_u16(B.fluxmoe_paged_tensor_address(pt, at_layer, 2, e), H * F)
                if not (torch.equal(a.cpu(), dense[weights_of][0][e].reshape(-1).view(torch.int16)) and
                        torch.equal(b.cpu(), dense[weights_of][1][e].reshape(-1).view(torch.int16))):
                    return False
            return True

        materialize(0)
        materialize(1)
        assert layer_shows(0, 0) and layer_shows(1, 1)
        assert layer_shows(2, 0) and layer_shows(3, 1)          # same parity, same physical block
        materialize(2)
        assert layer_shows(2, 2) and layer_shows(0, 2) and layer_shows(1, 1)

        # a kernel that takes plain dense pointers consumes expert 5 of layer 2 through its
        # virtual addresses (gate 1 for every token)
        x = inputs.activations(cfg, 2).cuda()
        out = torch.zeros((cfg.tokens, H), dtype=torch.float32, device="cuda")
        B.fluxmoe_shared_expert_ffn(ctx, B.fluxmoe_paged_tensor_address(pt, 2, 1, 5),
                                    B.fluxmoe_paged_tensor_address(pt, 2, 2, 5), x.data_ptr(), cfg.tokens,
                                    out.data_ptr())
        torch.cuda.synchronize()
        xb = inputs.bits_u16(x.cpu())
        w13b, w2b = inputs.bits_u16(dense[2][0][5]), inputs.bits_u16(dense[2][1][5])
        ref = offn.expert_ffn(offn.bf16_bits_to_f64(xb), offn.bf16_bits_to_f64(w13b),
                              offn.bf16_bits_to_f64(w2b), round_h=True)
        assert offn.rel_frobenius(out.cpu().numpy().astype(np.float64), ref) <= 1e-3

        # residency change: layer 2 becomes uncompressed-resident; same addresses, own block
        addr13 = B.fluxmoe_paged_tensor_address(pt, 2, 1, 0)
        B.fluxmoe_paged_tensor_set_class(pt, 2, True)
        assert B.fluxmoe_paged_tensor_address(pt, 2, 1, 0) == addr13
        info2 = B.fluxmoe_paged_tensor_info_get(pt)
        assert info2.n_uncompressed == 1 and info2.physical_bytes == 3 * (lay["S"][1] + lay["S"][2])
        for e in range(L):
            write_u16(B.fluxmoe_paged_tensor_address(pt, 2, 1, e), dense[2][0][e].reshape(-1).view(torch.int16).cuda())
            write_u16(B.fluxmoe_paged_tensor_address(pt, 2, 2, e), dense[2][1][e].reshape(-1).view(torch.int16).cuda())
        materialize(0)                                           # refills F_0
        assert layer_shows(0, 0) and layer_shows(2, 2)          # layer 2 no longer aliases F_0
        B.fluxmoe_paged_tensor_set_class(pt, 2, False)
        assert layer_shows(2, 0)                                 # back on the reusable block
        assert B.fluxmoe_paged_tensor_info_get(pt).physical_bytes == info.physical_bytes
    finally:
        torch.cuda.synchronize()
        B.fluxmoe_destroy(ctx)
        B.fluxmoe_paged_tensor_destroy(pt)


def test_padding_when_the_layer_group_is_not_a_multiple_of_the_granularity():
    # sigma_2 = 8 * 24 * 2 = 384 B, L = 3: A_2 = 1152, A_1 = 2304; every granularity pads them
    pt = B.fluxmoe_paged_tensor_create(3, 3, 8, 24, uncompressed=[0, 1, 0])
    try:
        info = B.fluxmoe_paged_tensor_info_get(pt)
        lay = opg.paged_tensor_layout(3, 3, 8, 24, info.granularity, 1)
        assert info.pad_bytes == lay["M_pad"] > 0 and info.physical_bytes == lay["physical"]
        a = B.fluxmoe_paged_tensor_address(pt, 2, 2, 2)
        assert a == info.v0[1] + 2 * lay["S"][2] + 2 * 384
        t = torch.arange(192, dtype=torch.int16, device="cuda")
        write_u16(a, t)
        assert torch.equal(read_u16(a, 192), t)
        # layers 0 and 2 share F_0; layer 1 has its own block
        assert torch.equal(read_u16(B.fluxmoe_paged_tensor_address(pt, 0, 2, 2), 192), t)
    finally:
        B.fluxmoe_paged_tensor_destroy(pt)
