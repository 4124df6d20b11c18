"""pytest plugin (`-p replay_plugin`) that lets the GPU parity test files run on a machine without a GPU:
the binding loads the host-model build of the library (tests/host_model/build.sh --shared) instead of
libmxfp8.so, and placing tensors on "cuda" becomes a no-op, so the very same test code drives the very
same kernel sources on the CPU execution model. Used by tests/test_host_model_replay.py; it checks the
test code and the kernels' logic, not the hardware (timing, the matrix instruction's internal rounding)."""
import os
import types

import torch

import paper_2506_08027_amd.binding as binding

binding.LIB_PATH = os.environ["MXFP8_HOSTMODEL_LIB"]
binding._need_cuda = lambda *tensors: None
binding._stream = lambda stream: None
torch.Tensor.cuda = lambda self, *a, **k: self
torch.cuda.synchronize = lambda *a, **k: None
torch.cuda.current_stream = lambda *a, **k: types.SimpleNamespace(cuda_stream=0)


def _on_cpu(fn):
    def wrapped(*args, **kwargs):
        if str(kwargs.get("device", "")).startswith("cuda"):
            kwargs["device"] = "cpu"
        return fn(*args, **kwargs)
    return wrapped


for _name in ("empty", "zeros", "ones", "full", "tensor"):
    setattr(torch, _name, _on_cpu(getattr(torch, _name)))
