"""Scheduler-driven serving loop on the GPU (small): batches come from the doubling-budget scheduler, pages
from the pool's free list; finished requests' caches are read back and compared bit for bit inside the loop."""
import argparse
import io
import json
from contextlib import redirect_stdout

import pytest

pytestmark = pytest.mark.gpu


def test_serving_loop_small_both_policies():
    import bench
    buf = io.StringIO()
    with redirect_stdout(buf):
        bench.main_serve(argparse.Namespace(serve_requests=10))
    lines = [json.loads(l) for l in buf.getvalue().splitlines() if l.startswith("{")]
    assert [l["config"]["policy"] for l in lines] == ["db", "mixed"]
    for l in lines:
        assert l["caches_checked_bit_exact"] >= 1
        assert l["generated_tokens"] == lines[0]["generated_tokens"] > 0
    assert lines[1]["iterations"] < lines[0]["iterations"]      # mixed launches need fewer iterations
