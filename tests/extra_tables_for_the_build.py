"""Table sets of a caller's own, as LLMEM_BUILD_TABLES hands them to the build step (used by
test_library_host.py; not a test module)."""
import numpy as np

from workloads import tables as T


def more():
    mine = T.random_table(np.random.default_rng(3), 10, 40, "mine", n_sizes=6)
    return [("mine", [mine]), ("mine_and_gpt", [mine, T.gpt_table()])]


def repeated():
    return [("llama", [T.llama_table()])]
