"""The measured-traffic table bench.py reads (profiles/hbm_traffic_table.txt) must belong to the library that
is built: a kernel change comes with a new nova_version() and a fresh collection, or the headline run would
report no traffic figure."""
import importlib.util
import os

from paper_2512_18453_amd import nova, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_table_covers_the_built_library():
    bench = load_bench()
    version = nova.nova_version()
    # the headline workload: all three stage kernels
    for stage, algorithmic in (("input_transform", 131661824), ("contract", 253952000), ("output_transform", 211943424)):
        got = bench.measured_traffic(version, "vgg_conv3_f83_fp16", "nova", "f32", 32, stage)
        assert got is not None, (version, stage)
        assert 0.95 * algorithmic < got < 1.15 * algorithmic, (stage, got)       # no wasted re-reads
    # every single-layer workload has its dominant kernels in the table
    seen = set()
    with open(bench.TRAFFIC_TABLE) as fh:
        for line in fh:
            cells = [c.strip() for c in line.split("|")]
            if len(cells) == 7 and not line.startswith("#") and cells[0] == version:
                seen.add(cells[1])
    assert set(synth.LAYER_CONFIGS) <= seen, set(synth.LAYER_CONFIGS) - seen
    # a stale key yields nothing rather than an old figure
    assert bench.measured_traffic("libnova 0.0", "vgg_conv3_f83_fp16", "nova", "f32", 32, "contract") is None
