"""The byte and flop figures that bench.py divides by time (the roofline numerators), checked against what the
model shapes fix by hand arithmetic: every projection weight and norm vector once per decode step, each live
row's key/value history once, one new slot and one embedding row per live row."""
import importlib.util
import pathlib

from paper_2305_13144_amd import synth

_spec = importlib.util.spec_from_file_location("bench", pathlib.Path(__file__).resolve().parent.parent / "bench.py")
bench = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(bench)


def test_weight_bytes_per_decode_step_7b_and_13b():
    # 7B: per layer q,k,v,o 4*4096^2, gate,up,down 3*4096*11008, two norm vectors; head 32000*4096 + final norm; bf16
    per_layer_7b = (4 * 4096 * 4096 + 3 * 4096 * 11008 + 2 * 4096) * 2
    assert per_layer_7b == 404_766_720
    assert synth.LLAMA7B.weight_bytes_per_step() == 32 * per_layer_7b + (32000 * 4096 + 4096) * 2 == 13_214_687_232
    per_layer_13b = (4 * 5120 * 5120 + 3 * 5120 * 13824 + 2 * 5120) * 2
    assert synth.LLAMA13B.weight_bytes_per_step() == 40 * per_layer_13b + (32000 * 5120 + 5120) * 2 == 25_704_048_640


def test_kv_bytes_per_token():
    assert synth.LLAMA7B.kv_bytes_per_token() == 2 * 32 * 4096 * 2 == 524_288          # 512 KiB
    assert synth.LLAMA13B.kv_bytes_per_token() == 2 * 40 * 5120 * 2 == 819_200         # 800 KiB
    assert synth.TINY.kv_bytes_per_token() == 2 * 2 * 256 * 2 == 2_048                 # 2 KiB


def test_decode_step_bytes_is_weights_plus_history_plus_new_slot_plus_embedding():
    b = bench.decode_step_bytes(synth.LLAMA7B, 16, 200)
    assert b == 13_214_687_232 + 16 * 201 * 524_288 + 16 * 524_288 + 16 * 8_192 == 14_909_317_120
    # at the chip's 8 TB/s that is the 1.86 ms floor the 70 % target is quoted against
    assert abs(b / 8e12 * 1e3 - 1.864) < 1e-3
    # one more live row costs its history, its new slot and its embedding row
    assert bench.decode_step_bytes(synth.LLAMA7B, 17, 200) - b == 201 * 524_288 + 524_288 + 8_192


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: asking for more must end with a message and a non-zero status before anything
    touches a device."""
    import subprocess
    import sys
    root = pathlib.Path(__file__).resolve().parent.parent
    r = subprocess.run([sys.executable, str(root / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_roofline_traffic_comes_from_the_committed_counter_summary_or_is_null():
    """`roofline.traffic` is read from the committed rocprofv3 counter summary for exactly the shape and launch
    configuration it was taken at; for any other it is null with the reason, never a stale constant."""
    got, source = bench.profile_traffic("llama7b", 16, 200, 0)
    assert got is not None and source.startswith("profiles/decode_step_7b_hbm_traffic.txt")
    alg = bench.decode_step_bytes(synth.LLAMA7B, 16, 200)
    assert 1.0 <= got / alg < 1.10          # measured traffic: a few per cent above the algorithmic bytes, no re-reads
    for other in (("llama13b", 16, 200, 0), ("llama7b", 32, 200, 0), ("llama7b", 16, 100, 0), ("llama7b", 16, 200, 2)):
        got, why = bench.profile_traffic(*other)
        assert got is None and "another shape" in why
