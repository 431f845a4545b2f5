"""MI355X-native Block-attention prefill hot path (arXiv 2409.15355).

``paper_2409_15355_amd.binding`` is the thin ctypes face of the HIP library
(``ba_encode_blocks``, ``ba_reencode_positions``, ``ba_final_block_attention``);
``paper_2409_15355_amd.workloads`` holds the seeded synthetic inputs.  Importing
the package itself loads nothing.
"""
__all__ = ["binding", "workloads", "build"]
