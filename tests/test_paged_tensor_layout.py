"""PagedTensor sizes and addresses (Sec. 4.1): oracle pins and the library's host arithmetic."""
import numpy as np
import pytest

from oracle import paging as opg
from paper_2604_02715_amd import binding as B

MiB = 1 << 20


def test_evaluated_models_have_no_padding_at_2MiB_granularity():
    """Sec. 4.1: all evaluated models satisfy the VMM alignment requirement, M_pad = 0.  Rank-local
    shapes of Tab. "eval_model_memory" deployments: GLM-4.5 (EP 8: 20 experts per rank),
    Qwen3-Next (EP 4: 128), Mixtral (EP 2: 4 experts, or TP 2: 8 experts of half the ffn)."""
    for N, L_r, H, F in ((89, 20, 5120, 1536), (48, 128, 2048, 512), (32, 4, 4096, 14336), (32, 8, 4096, 7168)):
        lay = opg.paged_tensor_layout(N, L_r, H, F, 2 * MiB, n_uncompressed=5)
        assert lay["M_pad"] == 0 and lay["S"] == lay["A"]
        assert lay["sigma"][1] == 2 * lay["sigma"][2]                 # sigma_1 = 2 sigma_2 (Sec. 4.2)


def test_hand_numbers_with_padding():
    # L_r = 3, H = 8, F = 24: sigma_2 = 384 B, sigma_1 = 768 B; A = 1152 / 2304; g = 1024
    lay = opg.paged_tensor_layout(N=5, L_r=3, hidden=8, ffn=24, g=1024, n_uncompressed=2)
    assert lay["A"] == {1: 2304, 2: 1152} and lay["S"] == {1: 3072, 2: 2048}
    assert lay["M_pad"] == (2 + 2) * ((3072 - 2304) + (2048 - 1152))
    assert lay["virtual"] == 5 * (3072 + 2048) and lay["physical"] == 4 * (3072 + 2048)
    # first tensor of the first layer sits at v0; last expert of layer 4
    assert opg.paged_tensor_address(10_000, 2048, 384, 1, 1) == 10_000
    assert opg.paged_tensor_address(10_000, 2048, 384, 4, 3) == 10_000 + 3 * 2048 + 2 * 384
    assert [opg.reusable_block_of(i) for i in (1, 2, 3, 4)] == [0, 1, 0, 1]


def test_library_layout_matches_oracle():
    rng = np.random.Generator(np.random.Philox(3))
    for _ in range(300):
        N, L = int(rng.integers(1, 100)), int(rng.integers(1, 513))
        H, F = 8 * int(rng.integers(1, 700)), 8 * int(rng.integers(1, 2000))
        g = int(rng.choice([4096, 65536, 2 * MiB]))
        n_unc = int(rng.integers(0, N + 1))
        info = B.fluxmoe_paged_tensor_layout(N, L, H, F, g, n_unc)
        lay = opg.paged_tensor_layout(N, L, H, F, g, n_unc)
        assert [info.A[0], info.A[1]] == [lay["A"][1], lay["A"][2]]
        assert [info.S[0], info.S[1]] == [lay["S"][1], lay["S"][2]]
        assert info.pad_bytes == lay["M_pad"] and info.virtual_bytes == lay["virtual"]
        assert info.physical_bytes == lay["physical"]
        assert (info.n_uncompressed, info.n_pageable) == (n_unc, N - n_unc)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_paged_tensor_layout(4, 8, 256, 512, 0)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_paged_tensor_layout(4, 8, 256, 512, 4096, 5)
