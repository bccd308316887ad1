"""MI355X-native rank-order search: cost models over batches of rank orders (ring, halving-doubling, BCube,
double binary tree), multi-start 2-opt and pair-swap descents, integer simulated annealing, cost matrix from probes.

Thin binding over the C ABI in include/cc.h; the computation lives in csrc/*.hip."""
from .binding import (CC_COST_MAX, CC_MAX_N, CC_MOVES_2OPT, CC_MOVES_FLIP, CC_MOVES_OROPT, CC_RING_MAX, CC_RING_MAX_DIRECTED, CC_RING_SUM,  # noqa: F401
                      CC_RING_SUM_DIRECTED, EXPORTS, LIB_PATH, OBJECTIVES, CCError, SearchBuffers, cc_2opt_search,
                      cc_2opt_search_ex, cc_2opt_search_noalloc, cc_2opt_workspace_bytes, cc_bcube_cost_batch, cc_bcube_cost_batch_weighted,
                      cc_best_of_restarts, cc_cost_matrix_from_probes, cc_dbt_cost_batch, cc_init_tours, cc_local_search, cc_local_search_ex,
                      cc_rd_batch_workspace_bytes, cc_rd_cost_batch, cc_rd_swap_search, cc_rd_swap_search_ex, cc_ring_cost_batch,
                      cc_ring_cost_batch_u16, cc_ring_cost_batch_u8, cc_sa_rd_search, cc_sa_rd_search_ex, cc_sa_search, cc_sa_search_ex,
                      cc_status_string, cc_validate_matrix, cc_version, lib)
