"""A child process that looks profiled to the library (a profiler's tool library named in
LD_PRELOAD) and asks for kernels that would have to be built at run time."""
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROFILED_CHILD = """
import sys
sys.path.insert(0, %r)
import numpy as np, torch
import paper_2404_10933_amd as M
from workloads import tables as T
rng = np.random.default_rng(3)
t = T.random_table(rng, 12, 40, "t", n_sizes=6)
on_gpu = %r
device = "cuda" if on_gpu else "cpu"
cfg = M.DeviceConfigs.empty(64, device=device)
out = torch.empty(64, dtype=torch.int64, device=device)
if on_gpu:
    M.llmem_grid_generate(4, 0, 0, 64, cfg)
import ctypes
lib = M.load_library()
for kernel in (5, 6):
    tab = M.Tables([t], kernel=kernel, device=device if on_gpu else None)
    # straight through the C ABI (the binding would ask torch for a stream, which needs a GPU)
    rc = lib.llmem_estimate_ex(ctypes.byref(cfg.struct), 64, ctypes.byref(tab.struct), ctypes.c_void_p(out.data_ptr()), None, None)
    text = M.llmem_strerror(rc)
    assert rc == -4 and "LLMEM_KERNEL_CACHE" in text and "LD_PRELOAD" in text, (rc, text)
if on_gpu:
    M.llmem_estimate_ex(cfg, M.Tables([T.llama_table()], kernel=5), out, None)     # built in: no compiler needed
    M.llmem_estimate_ex(cfg, M.Tables([t], kernel=0), out, None)                   # the interpreting forms still run
    torch.cuda.synchronize()
print("ok")
"""


def run_profiled_child(on_gpu):
    import subprocess
    import sys
    # a name that cannot be loaded: the dynamic loader says so and goes on, the library sees the name
    preload = (os.environ.get("LD_PRELOAD", "") + " /nonexistent/librocprofiler-sdk-tool.so").strip()
    env = dict(os.environ, LD_PRELOAD=preload)
    env.pop("LLMEM_KERNEL_CACHE", None)
    out = subprocess.run([sys.executable, "-c", PROFILED_CHILD % (ROOT, on_gpu)], capture_output=True, text=True,
                         timeout=300, env=env)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
