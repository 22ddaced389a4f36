"""The benchmark's command line on a machine without a GPU: what must hold before any
kernel runs (one GPU only, the power sensor helper, the JSON contract's constants)."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_count_is_the_networks():
    import synth
    macs = sum(cout * ((h + 2 * p - k) // s + 1) ** 2 * cin * k * k for _, cin, cout, k, s, p, h in synth.conv_layers())
    b = _bench()
    assert macs == 832_667_936 and b.FLOP_PER_IMAGE == 2 * macs
    assert b.FP32_MFMA_PEAK_TFLOPS == 157.3 and b.HBM_PEAK_GBS == 8000.0


def test_power_sampling_reads_a_sensor_file(tmp_path):
    b = _bench()
    sensor = tmp_path / "power1_input"
    sensor.write_text("250000000\n")                     # microwatts
    calls = []
    got = b.sample_power(str(sensor), 0.05, lambda: calls.append(1), settle=0.02)
    assert abs(got["mean_w"] - 250.0) < 1e-9 and got["samples"] >= 1 and len(calls) >= got["samples"]
    missing = b.sample_power(str(tmp_path / "nothing"), 0.02, lambda: None)
    assert missing["samples"] == 0 and missing["mean_w"] != missing["mean_w"]     # NaN: no reading, no crash


def test_second_network_layer_list_is_consistent():
    import synth
    layers = synth.second_network_layers()
    assert [l[3] for l in layers] == [11, 5, 3, 3, 3]
    h = 227
    for i, (name, cin, cout, k, s, p, hin) in enumerate(layers):
        assert hin == h, name
        ho = (hin + 2 * p - k) // s + 1
        h = (ho - 3) // 2 + 1 if i in (0, 1) else ho      # 3x3 stride-2 pooling follows the first two layers
        if i + 1 < len(layers):
            assert layers[i + 1][1] == cout
