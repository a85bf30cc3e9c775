"""The oracle against hand-worked traces on 2-4 agent grids (tests/golden)."""
import pytest

import trace_runner
from oracle_backend import OracleTraceEnv

TRACES = trace_runner.load_traces()


@pytest.mark.parametrize("trace", TRACES, ids=[t["name"].split()[0] for t in TRACES])
def test_hand_trace(trace):
    trace_runner.run_trace(OracleTraceEnv, trace)
