"""Child process of test_first_decode_call_of_a_process_inside_a_capture: the first decode call this
process makes is made inside a stream capture; prints OK when two replays reproduce an eager call."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import numpy as np
import torch
from test_gpu_parity import DEV, FAST, Layer, f64, kv, synth

w = FAST.with_(name="fast_graph_cold", index=48, n_images=4)
L = Layer(w, 103)
L.compress()
q, kn, vn = synth.make_step_inputs(w, 0, 0)
gq, gkn, gvn = q.to(DEV), kn.to(DEV), vn.to(DEV)
s = torch.cuda.Stream()
g = torch.cuda.CUDAGraph()
with torch.cuda.stream(s):
    with torch.cuda.graph(g, stream=s):
        kv.kvc_reconstruct_attend_decode(L.shape, L.params, gq, L.gKc, L.gVc, L.gKt, L.gVt, w.text_len,
                                         w.text_cap, gkn, gvn, 0.0, L.out, L.lse, L.ws, stream=s)
torch.cuda.synchronize()
g.replay()
torch.cuda.synchronize()
first = f64(L.out).copy()
eager, _ = L.decode(gq, w.text_len, gkn, gvn)
L.out.zero_()
torch.cuda.synchronize()
g.replay()
torch.cuda.synchronize()
second = f64(L.out).copy()
print("OK" if np.array_equal(first, eager) and np.array_equal(second, eager) else "MISMATCH", flush=True)
