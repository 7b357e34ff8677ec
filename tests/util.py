"""Helpers shared by the GPU parity tests: run the HIP path through the binding, compare with the oracle."""
from __future__ import annotations

import numpy as np

from paper_2505_17412_amd import inputs

from oracle.compare import TOL, TOPK_MARGIN, assert_close, check_topk, rel_errors  # noqa: F401

# device plumbing (no arithmetic) lives in the package, so that bench.py and the smoke run do not import the test tree
from paper_2505_17412_amd.harness import GpuRun, build_blocks_gpu, params_of, run_gpu, to_dev, to_np  # noqa: E402,F401
