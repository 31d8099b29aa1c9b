"""MVUE N:M pruning of neural gradients + sparse update GEMM for MI355X (gfx950).

``api`` is the thin binding of the C ABI (``include/nm_mvue.h``); ``synth`` draws the seeded
synthetic workloads; ``build`` compiles the HIP library in-tree.
"""
from . import synth  # noqa: F401
from .api import (NmError, alloc_compressed, alloc_compressed_q8, load, mvue_prune_1of2, mvue_prune_1of4, mvue_prune_2of4,  # noqa: F401
                  mvue_prune_2of4_t, mvue_prune_1of2_t,
                  mvue_prune_2of4_q8, mvue_prune_1of2_q8, mvue_prune_2of4_q8_t, mvue_prune_1of2_q8_t, mvue_prune_4of8_approx, mvue_prune_producer, nm_cast_e4m3, nm_compress, nm_prune_greedy, nm_q8_scale, nm_rw_mix_probe, nm_update_gemm, nm_update_gemm_q8, nm_update_gemm_q8_shifted, nm_update_gemm_q8_workspace,
                  nm_update_gemm_shifted, nm_update_gemm_static, nm_update_gemm_static_max, nm_update_gemm_workspace)
