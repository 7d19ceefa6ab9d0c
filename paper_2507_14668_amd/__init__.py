"""MI355X-native Tensor-Train embedding-bag hot path (HIP kernels behind a C ABI)."""
from .binding import (Plan, Prof, Table, alloc_batch_desc, tt_core_sgd_update_batched,  # noqa: F401
                      tt_emb_bag_backward_batched, tt_emb_bag_forward_batched, tt_index_reorder_batched, TTError, alloc_workspace, load_library, tt_core_sgd_update,  # noqa: F401
                      tt_emb_bag_backward, tt_emb_bag_backward_sgd, tt_emb_bag_forward, tt_emb_bag_forward_static, tt_emb_bag_forward_sample, tt_reuse_buffer_bytes, tt_index_graph_edges, tt_bf16_cores_bytes, tt_cores_to_bf16, tt_emb_bag_forward_bf16, tt_index_reorder, tt_plan_status, FusedLayout, FusedTables, fusion_groups,
                      tt_workspace_bytes)
from .module import TTEmbeddingBag, TTEmbeddingBagCollection, TTFusedEmbeddingBags  # noqa: F401,E402
from .bijection import build_index_bijection, prefix_reuse_stats  # noqa: F401,E402
