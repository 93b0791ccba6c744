"""MI355X-native clustered sparse attention (AdaCluster hot path).

The compute lives in a C-ABI shared library built from the HIP sources under
`csrc/`; `binding` marshals torch device pointers into it.  `workloads` draws
the seeded synthetic inputs.  Nothing here falls back to a CPU path.
"""
__all__ = ["binding", "workloads", "build"]
