"""optstage: one pipeline stage of LLM training (F / B / W + activation offload / reload under an HBM
budget, executed in the order of a per-stage schedule) on one MI355X.  `binding` mirrors the C-ABI of
liboptstage.so one to one; `stage.Stage` obtains memory and streams from PyTorch and calls it."""
from . import binding  # noqa: F401
