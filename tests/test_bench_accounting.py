"""Host-side checks of the benchmark's bookkeeping: algorithmic work figures and the profile summariser (no GPU)."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import synth_inputs as si  # noqa: E402


def test_forward_backward_flop_count_of_the_workloads():
    """3 x forward, 2 M N K per projection, causal attention at half of 4 B H' N^2 d_head (Appendix A.1-A.2 shapes):
    the hand-computed totals of the five workload shapes, in TFLOP."""
    tf = lambda cfg, hs, fs, B, N: bench.flops_fwd_bwd(cfg, hs, fs, B, N) / 1e12
    assert abs(tf(si.CFG2, 3, 768, 8, 1024) - 3.06) < 0.005          # GPT-2-small quarter-width subnet (vocabulary projection: 62 %)
    assert abs(tf(si.CFG3, 8, 2816, 4, 2048) - 33.27) < 0.005        # Llama-1B half-width subnet: the bench step
    assert abs(tf(si.CFG3, 16, 5632, 4, 2048) - 63.32) < 0.005       # the same model at full width
    assert abs(tf(si.CFG5, 16, 5504, 2, 4096) - 178.8) < 0.05        # 7B shape pruned to half
    assert abs(tf(si.CFG5, 32, 11008, 2, 4096) - 351.1) < 0.05       # unpruned
    # one layer of the bench step by hand: QKV 103.1 + O 34.4 + gate/up 189.0 + down 94.5 + attention 34.4 GFLOP forward
    one = bench.flops_fwd_bwd(si.CFG3, 8, 2816, 4, 2048) - bench.flops_fwd_bwd(__import__("dataclasses").replace(si.CFG3, n_layers=21), 8, 2816, 4, 2048)
    assert abs(one / 3e9 - (103.08 + 34.36 + 188.98 + 94.49 + 34.36)) < 0.05


def test_profile_summariser_modes(tmp_path):
    from paper_2511_03983_amd import profile_summary as ps
    stats = tmp_path / "s.csv"
    stats.write_text('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
                     '"void (anonymous namespace)::pp::gemm_pp_kernel<1, 1, false>(int, int)",10,1000000,100000,80.0,1,2,0\n'
                     '"at::native::foo(int)",5,250000,50000,20.0,1,2,0\n')
    out = tmp_path / "s.txt"
    ps.stats(str(stats), str(out), "cmd")
    text = out.read_text()
    assert "pp::gemm_pp_kernel<1, 1, false>" in text and "other: at::native::foo" in text and "# command: cmd" in text
    pmc = tmp_path / "c.csv"
    rows = ['"Dispatch_Id","Kernel_Name","Grid_Size","Counter_Name","Counter_Value"']
    for d in (1, 2):
        for part in range(4):                               # a dispatch's counter arrives in several rows: they are summed
            rows.append(f'{d},"k1(int)",256,"FETCH_SIZE",{10.0 * d}')
        rows.append(f'{d},"k1(int)",256,"SQ_VALU_MFMA_BUSY_CYCLES",{3200.0}')
        rows.append(f'{d},"k1(int)",256,"SQ_BUSY_CYCLES",{200.0}')
        rows.append(f'{d},"k1(int)",256,"SQ_INSTS_VALU_MFMA_MOPS_BF16",{64.0}')
    pmc.write_text("\n".join(rows) + "\n")
    out2 = tmp_path / "c.txt"
    ps.pmc(str(pmc), str(out2), "cmd")
    line = [l for l in out2.read_text().splitlines() if l.startswith("k1") and "FETCH_SIZE" in l][0]
    assert line.split()[-2:] == ["2", "60.0"]               # two dispatches, (40 + 80) / 2 per dispatch
    out3 = tmp_path / "m.txt"
    ps.mfma(str(pmc), str(out3), "cmd")
    line = [l for l in out3.read_text().splitlines() if l.startswith("k1")][0]
    assert line.split()[-1] == "0.500"                      # 6400 / (32 x 400)
