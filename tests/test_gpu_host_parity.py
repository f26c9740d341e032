"""The host-side parity tests (batch formation, quad-tree + Density First
Search, batch-level scheduler: C ABI against the oracles, bit-exact) once more
under the `gpu` marker, so that the run on the GPU machine exercises them against
the library as it was loaded there.  The test bodies are the ones of
tests/test_abi.py, tests/test_quadtree_abi.py and tests/test_scheduler_abi.py;
nothing here needs the GPU itself."""
import pytest

from tests import test_abi as _abi
from tests import test_quadtree_abi as _qt
from tests import test_scheduler_abi as _sc

pytestmark = pytest.mark.gpu

# a1: as_aligned_batch against oracle/batcher.py
test_library_exports = _abi.test_library_loads_and_exports_every_declared_symbol
test_aligned_batch_bit_exact = _abi.test_aligned_batch_matches_oracle_bit_exact
test_aligned_batch_config_lengths = _abi.test_aligned_batch_on_the_config_lengths
test_aligned_batch_errors = _abi.test_aligned_batch_errors
test_attention_argument_errors = _abi.test_decode_attention_argument_errors_before_any_gpu_work
test_workspace_size_query = _abi.test_workspace_size_query

# Section 3.3, Algorithm 1: as_qtree_* / as_dfs_batches against oracle/quadtree.py
test_qtree_hand_worked = _qt.test_hand_worked_scenarios_through_the_abi
test_qtree_random = _qt.test_random_inputs_match_oracle
test_qtree_updates_and_starvation = _qt.test_interleaved_updates_and_starvation_match_oracle
test_qtree_errors = _qt.test_errors
test_qtree_benchmark_lengths = _qt.test_generator_on_the_benchmark_lengths

# Section 3.4, Algorithm 2: as_sched_* against oracle/decode_loop.py
test_sched_hand_worked = _sc.test_hand_worked_traces_through_the_abi
test_sched_random = _sc.test_random_traces_match_oracle
test_sched_errors = _sc.test_scheduler_errors
