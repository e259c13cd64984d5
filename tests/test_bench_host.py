"""Host logic of bench.py that needs no GPU: the algorithmic byte model and the look-up of the stored counter
traffic (it must be handed out only for the command line and the kernel sources it was measured with)."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_source_digest_is_stable_and_covers_the_kernel_sources():
    a, b = bench.source_digest(), bench.source_digest()
    assert a == b and re.fullmatch(r"[0-9a-f]{16}", a)


def test_stored_traffic_is_keyed_on_command_line_and_sources():
    for wl in ("C3", "C4"):
        path = os.path.join(ROOT, "profiles", "estep_kernel_%s_hbm_traffic.md" % wl)
        text = open(path).read()
        args = re.search(r"^bench_args = --steps (\d+) --warmup (\d+)$", text, flags=re.M)
        digest = re.search(r"^source_digest = ([0-9a-f]+)$", text, flags=re.M)
        value = re.search(r"^traffic_bytes_per_launch = (\d+)$", text, flags=re.M)
        assert args and digest and value, path
        steps, warmup = int(args.group(1)), int(args.group(2))
        got = bench.profiled_traffic(wl, steps, warmup)
        if digest.group(1) == bench.source_digest():
            assert got == float(value.group(1))
        else:
            assert got is None                      # measured on other kernel sources: not reported
        assert bench.profiled_traffic(wl, steps + 1, warmup) is None
        assert bench.profiled_traffic(wl, steps, warmup + 1) is None
    assert bench.profiled_traffic("C1", 20, 5) is None      # no summary stored for this workload


def test_algorithmic_bytes_model():
    """Per token 20 bytes (16-bit assignments); per run its row once; per (word, chunk) and iteration the tree level,
    block bases and total plus the row (dense: 4 Kpad; light: 8 + 8 per non-zero); the base vector once per
    iteration: the list in bench.algorithmic_bytes, evaluated by hand on a made-up statistics record."""
    st = {"sum_tokens": 1000, "sum_row_fetch": 5000, "words_present": 10, "light_words_present": 4, "sum_light_entries": 30,
          "iterations": 2}
    K, Kpad, n3, n3pad = 100, 128, 2, 64
    tree = 4 * n3pad + 8 * n3 + 4
    want = 1000 * (4 + 4 + 8 + 2 * 2) + 5000 * 4                    # tokens and rows of A
    want += 2 * 6 * (4 * Kpad + tree)                               # six dense-row words, two iterations
    want += 2 * 4 * (8 + tree) + 30 * 8                             # four light words, 30 non-zeros staged in all
    want += 2 * 4 * Kpad                                            # the base vector
    assert bench.algorithmic_bytes(st, K, 2) == want
    st["light_words_present"] = 0; st["sum_light_entries"] = 0
    assert bench.algorithmic_bytes(st, K, 4) == 1000 * 24 + 5000 * 4 + 2 * 10 * (4 * Kpad + tree)
