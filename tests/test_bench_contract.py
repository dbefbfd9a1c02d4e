"""bench.py's contract on the CPU: more than one GPU is refused with a message
(this build uses one), and the work models behind the reported figures count what
their comments say."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stderr + res.stdout) and "--gpus 1" in (res.stderr + res.stdout)
    assert not any(line.startswith("{") for line in res.stdout.splitlines())      # no result line


def test_recorded_fullsize_oracle_time_is_read():
    b = load_bench()
    rec = b.recorded_fullsize_oracle()
    assert rec and rec["SECONDS"] > 60 and rec["CORES"] >= 1


def test_work_models():
    b = load_bench()
    D, N = 1 << 25, 1 << 16
    # the headline's model: ten multiplications per tensor entry and per table row
    assert b.fr_mul_model(D, N) == 10 * D + 10 * N
    # the dominant kernel runs the rounds before the table's variables, above 256 pairs, after the first round -- or, from
    # a vector of field elements, after the first two, which share the first pass
    assert b.first_two_rounds_share_a_pass(D, N)
    assert b.rounds_on_29_bits(D, N) == list(range(2, 9)) and b.rounds_on_29_bits(D, N, from_ints=True) == list(range(1, 9))
    pairs, muls, moved = b.round29_work(D, N)
    assert pairs == sum(D >> (k + 1) for k in range(2, 9)) == D // 4 - D // 512
    # round 2 binds two variables (17 multiplications, 20 entries per pair), rounds 3..8 one (9 and 12)
    assert muls == 17 * (D >> 3) + 9 * (D // 8 - D // 512) and moved == 32 * (20 * (D >> 3) + 12 * (D // 8 - D // 512))
    assert b.rounds_on_29_bits(1 << 12, 1 << 4) == [2]               # 512 pairs; 256 is the resident kernel's
    assert b.rounds_on_29_bits(1 << 12, 1 << 4, from_ints=True) == [1, 2]
    assert b.rounds_on_29_bits(1 << 12, 1 << 11) == []               # the table's variables start at the second round
    assert b.rounds_on_29_bits(1 << 12, 1 << 10) == [1]              # ... at the third: no pass can serve two rounds
    # nine multiplications of 112 multiply-adds per pair against 256 CUs x 64 lanes x 2.4 GHz
    assert (b.ROUND_DATA_FR_MUL_PER_PAIR_EVAL + b.ROUND_DATA_FR_MUL_PER_PAIR_FOLD, b.MADS_PER_FR_MUL) == (9, 112)
    assert b.PEAK_MAD_PER_S == 256 * 64 * 2.4e9
    # the whole prove against the HBM roof: 292 bytes per element that must move even with perfect fusion, 8 TB/s
    assert (b.WHOLE_PROVE_BYTES_PER_ELEMENT, b.PEAK_HBM_BYTES_PER_S) == (4 + 96 + 192, 8e12)
    # the linking sumcheck: 11, 15, then 13 multiplications per pair, and one per entry for each digit tensor's value
    Dl = 1 << 10
    assert b.link_fr_mul_model(Dl) == 11 * (Dl // 2) + 15 * (Dl // 4) + 13 * (Dl // 4 - 1) + 2 * Dl
