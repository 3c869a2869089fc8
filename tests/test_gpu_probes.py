"""The measurement probes of the boundary (sr_probe_*): they reject what they do not support, and what they report on
an MI355X lies where the chip's published figures allow.  They are auxiliaries of the roofline report, not steps of
the rollout path, so there is no checker value to compare with: the tests are argument checks and sanity ranges."""
import pytest
import torch

import paper_2605_05802_amd as sr

pytestmark = pytest.mark.gpu


def expect_arg_error(fn, *a, **k):
    with pytest.raises(sr.SrError) as e:
        fn(*a, **k)
    assert e.value.status == sr.SR_E_ARG


def test_streaming_read_and_copy_rates_are_plausible_and_bad_arguments_are_refused():
    src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")          # 1 GiB
    dst = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
    nt, plain, copy = (sr.sr_probe_hbm(src, dst, m) for m in (0, 1, 2))
    print(f"read (non-temporal) {nt:.0f} GB/s, read {plain:.0f} GB/s, copy {copy:.0f} GB/s")
    for v in (nt, plain, copy):
        assert 2000 < v < 8000                                             # below the published 8 TB/s, well above PCIe
    expect_arg_error(sr.sr_probe_hbm, src, dst, 3)
    expect_arg_error(sr.sr_probe_hbm, src, None, 2)
    tiny = torch.zeros(1024, dtype=torch.int32, device="cuda")
    expect_arg_error(sr.sr_probe_hbm, tiny, dst, 0)                        # less than one run per wavefront


def test_matrix_loop_rate_is_plausible_and_loads_beside_it_cost_something():
    scratch = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    buf = torch.zeros(1 << 18, dtype=torch.int32, device="cuda")           # 1 MiB
    alone = sr.sr_probe_mfma_bf16(scratch)
    assert 1000 < alone < 2600                                             # TFLOP/s; the published dense peak is 2500
    free, _ = sr.sr_probe_mfma_under_loads(buf, scratch, 0, 0)
    lds4, lds4_rate = sr.sr_probe_mfma_under_loads(buf, scratch, 2, 4)
    reg4, reg4_rate = sr.sr_probe_mfma_under_loads(buf, scratch, 1, 4)
    print(f"matrix loop {alone:.0f} TFLOP/s; eight wavefronts per CU {free:.0f}; with 4 loads per 16 MFMAs straight into "
          f"LDS {lds4:.0f} ({lds4_rate:.0f} GB/s), into registers {reg4:.0f} ({reg4_rate:.0f} GB/s)")
    assert 1000 < free < 2600 and 300 < lds4 < free and 300 < reg4 < free
    assert 1000 < lds4_rate < 40000 and 1000 < reg4_rate < 40000
    expect_arg_error(sr.sr_probe_mfma_under_loads, buf, scratch, 1, 3)     # unsupported number of loads
    expect_arg_error(sr.sr_probe_mfma_under_loads, buf, scratch, 0, 4)     # loads without a path
    expect_arg_error(sr.sr_probe_mfma_under_loads, buf, scratch, 1, 4, True)
    expect_arg_error(sr.sr_probe_mfma_under_loads, buf, scratch, 3, 4)
    odd = torch.zeros(3 << 16, dtype=torch.int32, device="cuda")           # not a power of two
    expect_arg_error(sr.sr_probe_mfma_under_loads, odd, scratch, 2, 4)
    small = torch.zeros(1024, dtype=torch.float32, device="cuda")          # scratch too small
    expect_arg_error(sr.sr_probe_mfma_under_loads, buf, small, 2, 4)


def test_decode_attention_probe_phases_and_merge():
    shared, nbytes_s = sr.sr_probe_decode_attention(16, 8, 1024, 1000, 2, 1, False, 8)
    both, nbytes_b = sr.sr_probe_decode_attention(16, 8, 1024, 1000, 2, 3, False, 8)
    merged, _ = sr.sr_probe_decode_attention(16, 8, 1024, 1000, 2, 7, False, 8)
    print(f"shared phase {shared:.1f} us, both {both:.1f} us, with the merge launch {merged:.1f} us")
    assert nbytes_s == 16 * 1024 * 2048 and nbytes_b == nbytes_s + 128 * 1000 * 2048
    assert 0 < shared < both < merged < 1000
    expect_arg_error(sr.sr_probe_decode_attention, 16, 8, 1024, 1000, 2, 0)
    expect_arg_error(sr.sr_probe_decode_attention, 16, 8, 1024, 1000, 2, 4)     # a merge of nothing
    expect_arg_error(sr.sr_probe_decode_attention, 16, 8, 1000, 1000, 2, 3)     # prompt not in whole pages
    expect_arg_error(sr.sr_probe_decode_attention, 16, 8, 0, 1000, 2, 1)        # no shared prompt to time
    expect_arg_error(sr.sr_probe_decode_attention, 16, 1, 1024, 1000, 2, 3)     # a group is at least two members
