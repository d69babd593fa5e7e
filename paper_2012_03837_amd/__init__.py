"""Local-parallelism training step for AMD MI355X: HIP kernels behind a C ABI (liblp.so) and a thin
ctypes binding with the same entry-point names."""
from .binding import (LpError, LocalTrainer, lib, make_spec, lp_query_sizes, lp_init_blocks, lp_local_step,
                      lp_eval_loss, lp_tensor_info, lp_get_tensor, lp_set_tensor, lp_param_names, lp_get_step,
                      lp_set_step, lp_destroy, lp_profile_enable, lp_profile_read, lp_profile_gemm_shapes, lp_profile_gemm_kernels, lp_cost_model, lp_mlp_flops, lp_grad_cosine, lp_step_graph, lp_bn_running, lp_overlap_steps, lp_join, default_side_streams,
                      METHODS, KERNEL_CLASSES, LIB_PATH)

__all__ = ["LpError", "LocalTrainer", "lib", "make_spec", "lp_query_sizes", "lp_init_blocks", "lp_local_step",
           "lp_eval_loss", "lp_tensor_info", "lp_get_tensor", "lp_set_tensor", "lp_param_names", "lp_get_step",
           "lp_set_step", "lp_destroy", "lp_profile_enable", "lp_profile_read", "lp_profile_gemm_shapes", "lp_profile_gemm_kernels", "lp_cost_model", "lp_mlp_flops", "lp_grad_cosine", "lp_step_graph", "lp_bn_running", "lp_overlap_steps", "lp_join", "default_side_streams", "METHODS", "KERNEL_CLASSES", "LIB_PATH"]
