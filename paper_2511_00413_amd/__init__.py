"""MI355X-native tree-attention hot path of Tree Training: thin Python binding over the C ABI in
include/treetrain.h.  Every step runs in the HIP library; this package only marshals arguments
(torch tensors supply device memory and the stream).  There is no CPU fallback: if the shared
library is missing, importing the binding raises."""
from .binding import (  # noqa: F401
    TreeMeta, TreeTrainError, lib_path, tree_attn_bwd, tree_attn_fwd, tree_attn_workspace,
    tree_build_meta, tree_meta_sizes, tree_weighted_logprob, tree_weighted_logprob_bwd, tree_weighted_logprob_fwd_bwd, tree_rope, last_error, version, KTILE,
    kernel_timing_enable, kernel_timing_read, PartitionPlan, ConvPlan, GdnPlan, tree_gdn_plan, tree_gdn_fwd, tree_gdn_bwd, tree_gdn_bwd_workspace, GDN_CHUNK, tree_conv_plan, tree_conv_fwd, tree_conv_bwd, tree_conv_bwd_static, CONV_BWD_STATIC_SCRATCH_BYTES, tree_path_weights, WEIGHT_PATH_SUM, WEIGHT_UNIFORM, WEIGHT_PATH_TOKEN_MEAN,
    tree_partition_sizes, tree_partition_plan,
    tree_attn_partitioned_workspace, tree_attn_partitioned_fwd, tree_attn_partitioned_bwd,
)
