"""MI355X-native ShotKV KV-cache compression hot path (arXiv 2502.01941, Section 5, Algorithm 1).

`paper_2502_01941_amd.shotkv` is the thin binding over the C-ABI library built from `csrc/`;
`paper_2502_01941_amd.workloads` draws the seeded synthetic inputs.  Nothing is imported eagerly so
that the input generators can be used without the compiled library.
"""
__all__ = ["shotkv", "workloads"]
