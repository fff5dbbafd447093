"""First calls from two host threads at once (fresh process: nothing has set a kernel's per-device limits yet).
Each thread runs the bf16 matrix-core path -- forward, backward, selection -- on a stream of its own with
buffers of its own; both must reproduce the single-threaded results bit for bit."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCRIPT = r"""
import sys, threading
sys.path.insert(0, %r)
import torch
from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype

w = WORKLOADS["mid_sparse_bf16"]
api.lib()
results = [None, None]
start = threading.Barrier(2)

def work(idx):
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        x = make_inputs(w, "cuda")
        desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
        stream.synchronize()
        start.wait()                      # both threads make their first library calls together
        sel, cnt = api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k)
        o, lse = api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt)
        dq = api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                                x["dv_pool"], sel, cnt)
        stream.synchronize()
    results[idx] = [t.cpu() for t in (sel, cnt, o, lse, dq, x["dk_pool"], x["dv_pool"])]

threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
for t in threads: t.start()
for t in threads: t.join()
assert results[0] is not None and results[1] is not None, "a thread failed"
for a, b in zip(*results):
    assert torch.equal(a, b), "the two threads disagree"
# and against a plain single-threaded pass
x = make_inputs(w, "cuda")
desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
sel, cnt = api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k)
o, lse = api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt)
dq = api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"], x["dv_pool"], sel, cnt)
torch.cuda.synchronize()
for a, b in zip(results[0], (sel, cnt, o, lse, dq, x["dk_pool"], x["dv_pool"])):
    assert torch.equal(a, b.cpu()), "threaded and single-threaded results differ"
print("THREADS_OK")
"""


def test_first_calls_from_two_threads():
    out = subprocess.run([sys.executable, "-c", SCRIPT % ROOT], capture_output=True, text=True, timeout=240)
    assert out.returncode == 0 and "THREADS_OK" in out.stdout, out.stdout[-2000:] + out.stderr[-4000:]
