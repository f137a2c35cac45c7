"""Every micro-benchmark kind that include/hikonv_bench.h names launches and finishes (tiny sizes)."""
import pytest

pytestmark = pytest.mark.gpu


def test_every_ubench_kind_runs():
    import torch
    import paper_2208_00763_amd as hk
    valu = [hk.UB_MAD_U32_U24, hk.UB_MAD_U64_U32, hk.UB_MUL_LO_U32, hk.UB_BFE_U32, hk.UB_LSHR_B64, hk.UB_DPP_MOV,
            hk.UB_ADD_U32, hk.UB_MAD_I32_I24, hk.UB_MAD_I64_I32, hk.UB_ADD_U64, hk.UB_ALIGNBIT, hk.UB_AND_B32,
            hk.UB_ASHR_I64, hk.UB_BFE_I32, hk.UB_CHAIN_MAD_I64_I32, hk.UB_CHAIN_MAD_I32_I24]
    assert sorted(valu) == list(range(16))
    buf = torch.zeros(4 * 256, dtype=torch.int32, device="cuda")
    for kind in valu:
        hk.hikonv_ubench(kind, 2, 4, buf)
    torch.cuda.synchronize()
    big = torch.zeros(1 << 18, dtype=torch.int32, device="cuda")
    for kind in (hk.UB_HBM_WRITE, hk.UB_HBM_WRITE_NT, hk.UB_HBM_WRITE_RUNS):
        big.zero_()
        hk.hikonv_ubench(kind, 0, 64, big)
        torch.cuda.synchronize()
        assert int((big.view(-1, 4)[:, 2] == 3).sum()) == big.numel() // 4      # every 16-byte store landed
    for bits in (1, 2, 32):
        big.zero_()
        hk.hikonv_ubench(hk.UB_HBM_WRITE_VARIED, bits, 64, big)
        torch.cuda.synchronize()
        if bits < 32:
            assert int(big.max()) < (1 << bits) and int(big.min()) >= 0
        assert int((big != 0).sum()) > big.numel() // 4
    with pytest.raises(hk.HikonvError):
        hk.hikonv_ubench(hk.UB_HBM_WRITE_VARIED, 0, 64, big)
    with pytest.raises(hk.HikonvError):
        hk.hikonv_ubench(hk.UB_HBM_WRITE_VARIED, 33, 64, big)
    hk.hikonv_ubench(hk.UB_HBM_COPY, 0, 64, big)
    hk.hikonv_ubench(hk.UB_HBM_READ, 0, 64, big)
    torch.cuda.synchronize()
    assert torch.equal(big[: big.numel() // 2], big[big.numel() // 2:])       # copy: first half -> second
