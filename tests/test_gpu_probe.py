"""The MFMA probe (benchmark aid): every loop executes the MFMAs it claims.  On all-ones operands each
v_mfma_f32_32x32x16_bf16 adds 16 to every element of its accumulator, so the accumulators count the MFMAs."""
import pytest
import torch

import paper_2407_00611_amd as st

pytestmark = pytest.mark.gpu


def test_probe_loops_execute_the_mfmas_they_report():
    facts = st.st_device_facts()
    blocks = facts["compute_units"]
    ones = torch.ones(1 << 16, dtype=torch.bfloat16, device="cuda")
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    for mix in range(st.st_mfma_probe_mixes() + 1):
        for iters in (1, 3):
            sink.fill_(-1.0)
            flop = st.st_mfma_probe(ones, iters, sink, mix)
            torch.cuda.synchronize()
            mfmas = flop / (2.0 * 32 * 32 * 16) / (blocks * 4)          # per wavefront
            assert mfmas == int(mfmas) and mfmas % (4 * iters) == 0, (mix, iters, mfmas)
            # four accumulators take the MFMAs in turn; the MFMA-only loop sums all 16 values a lane holds of each
            # accumulator, the loops with side instructions one value of each
            per_value = 16.0 * mfmas / 4
            expect = per_value * 4 * (16 if mix == 0 else 1)
            assert bool((sink == expect).all()), (st.st_mfma_probe_mix_name(mix), iters, float(sink[0]), expect)


def test_probe_with_side_instructions_runs_on_arbitrary_data():
    """Side instructions read the operands as numbers (exponentials, packs, LDS reads): any bit pattern must do."""
    facts = st.st_device_facts()
    g = torch.Generator(device="cuda").manual_seed(7)
    bits = torch.randint(-32768, 32767, (1 << 18,), dtype=torch.int16, device="cuda", generator=g)
    sink = torch.empty(facts["compute_units"] * 256, dtype=torch.float32, device="cuda")
    for mix in range(1, st.st_mfma_probe_mixes() + 1):
        assert st.st_mfma_probe(bits.view(torch.bfloat16), 2, sink, mix) > 0
    torch.cuda.synchronize()
