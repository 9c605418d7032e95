"""MI355X-native pdADMM-G / pdADMM-G-Q iteration: thin ctypes binding over libpdadmm.so.

Every step of the method runs in the HIP library; this package only marshals arguments
(torch tensors -> raw pointers). There is no CPU fallback: a missing library is an error.
"""
from .binding import (PdadmmError, Config, Context, load_library, library_path, exported_symbols,
                      pdadmm_normalize_adj, pdadmm_augment, pdadmm_quantize, pdadmm_gemm_nt,
                      pdadmm_gemm_tn, pdadmm_gemm_tn_static, pdadmm_workspace_bytes, pdadmm_init, pdadmm_grow_layers,
                      pdadmm_set_var,
                      pdadmm_get_var, pdadmm_iterate, pdadmm_step_phase, pdadmm_sync,
                      pdadmm_objective, pdadmm_residual, pdadmm_stats, pdadmm_plan_info, pdadmm_predict, pdadmm_destroy,
                      pdadmm_timing, pdadmm_timing_read, TIMING_CLASSES,
                      VAR, PHASE, RISK, thread_error)

__all__ = [n for n in dir() if not n.startswith("_")]
