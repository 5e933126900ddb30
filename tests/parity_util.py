"""What the GPU parity tests share, under one name: moving a seeded problem to the GPU and back
(paper_2603_13420_amd/inputs.py: data only) and comparing a result with the CPU oracle under the
bounds derived from the kernels' arithmetic (oracle/parity.py, where the derivation is written out)."""
from oracle.parity import *                                                     # noqa: F401,F403
from oracle.parity import forward_bound, grad_bounds, eta_fp32                  # noqa: F401
from paper_2603_13420_amd.inputs import make_dout, out_to_f64, to_device, to_device_multi   # noqa: F401
