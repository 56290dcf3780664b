"""MI355X-native Contextual Token Sparsity hot path (LeMo, arXiv 2501.09767).

``paper_2501_09767_amd.lemo`` is the thin binding over the C-ABI HIP library
(``lemo_score_segments``, ``lemo_select_topk``, ``lemo_gather_gemm``, ``lemo_scatter_grad``);
``paper_2501_09767_amd.workloads`` builds seeded synthetic inputs.  Nothing is imported eagerly so
that the input generators can be used without the HIP library being present.
"""
__all__ = ["lemo", "workloads", "build"]
