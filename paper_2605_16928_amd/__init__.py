"""MI355X-native sparse-attention hot path of RTPurbo (indexer score, dynamic top-p,
sparse / local / dense attention) behind a C-ABI HIP library.

`paper_2605_16928_amd.rtp` is the thin ctypes binding (argument marshalling only);
`paper_2605_16928_amd.workloads` draws the seeded synthetic inputs.  The HIP
library is loaded on first use and its absence is an error: there is no CPU
fallback.
"""
__all__ = ["rtp", "workloads"]
