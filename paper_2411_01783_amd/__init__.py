"""MI355X-native per-rank hot path of context-parallel ring attention.

`paper_2411_01783_amd.binding` wraps the C-ABI library (libcp_attn.so, built
from csrc/ for gfx950); `paper_2411_01783_amd.workloads` draws the seeded
synthetic inputs. Importing the package loads neither torch kernels nor the
library; the binding loads the library on first use and raises if it is absent.
"""
__all__ = ["binding", "workloads"]
