"""MI355X-native hot path of FedRAG's Scrambled Distributed Attention (one node's share).

`paper_2605_25716_amd.binding` wraps the C-ABI library (include/fedrag.h) one-to-one;
`paper_2605_25716_amd.workloads` draws seeded synthetic inputs and keys.  Nothing is loaded
at import time; the binding raises if the HIP library has not been built.
"""
__all__ = ["binding", "workloads", "build"]
