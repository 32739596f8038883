"""libepara for MI355X: grouped dense forward of co-located inference services.

`binding` mirrors include/epara.h one to one (ctypes); `runtime` and `mixrun` marshal PyTorch
device memory into it.  The HIP library must be built (`python -m paper_2511_00603_amd.build`);
nothing here computes on the CPU.
"""
from . import binding  # noqa: F401
