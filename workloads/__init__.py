"""Seeded synthetic inputs for the Tag roll-out path (configs and policy outputs).

Serves both the CPU oracle's tests and the GPU path's tests and benchmark.  It
holds none of the method's arithmetic: only sizes, seeds and the stand-in for the
policy network's output (softmax of N(0,1) logits).
"""
from .tag import (CONFIGS, CTAG_CONFIGS, CTagConfig, TagConfig, ctag_probs_for_step, device_probs_ring,  # noqa: F401
                  probs_for_step)
