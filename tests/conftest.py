import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Collection order of the GPU files: the kernels a caller gets by default first, every other kernel family
# next, the reproduction of the paper's printed accuracy figures (a statement about error levels, not
# parity) near the end and the entry point that allocates nothing last, so that under `-x` a failure in a
# late file cannot hide the parity cases of the hot path.  Files not listed keep their alphabetical place
# ahead of the listed ones.
GPU_FILE_ORDER = [
    "test_gpu_parity.py",
    "test_gpu_parity_workers.py",
    "test_gpu_parity_scale_comp.py",
    "test_gpu_parity_lazy.py",
    "test_gpu_parity_y_long_context.py",
    "test_gpu_parity_t_graph.py",
    "test_gpu_parity_tables_3_4.py",
    "test_zz_no_alloc.py",
]


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(session, config, items):
    rank = {name: i + 1 for i, name in enumerate(GPU_FILE_ORDER)}
    items.sort(key=lambda it: rank.get(os.path.basename(str(it.fspath)), 0))   # stable: order inside a file is kept
