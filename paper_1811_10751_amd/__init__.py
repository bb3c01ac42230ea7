"""MI355X-native Generalized PolyDot coded computation (arXiv 1811.10751): thin Python
binding over the C-ABI library libgpd.so built from csrc/ (hand-written HIP, gfx950)."""
from .binding import *  # noqa: F401,F403
from .binding import (GpdError, Layer, Plan, Report, load_library, gpd_coded_layer_step, gpd_decode,
                      gpd_encode, gpd_host_code, gpd_host_decode_matrices, gpd_l2_delta,
                      gpd_layer_create, gpd_layer_decode_weights, gpd_layer_encode_weights, gpd_plan,
                      gpd_sigmoid_bwd, gpd_sigmoid_fwd, gpd_version, gpd_worker_products,
                      NodeReport, gpd_locate_nodes, gpd_layer_locate_nodes, gpd_layer_regenerate,
                      gpd_layer_project, gpd_host_parity_check, gpd_host_locate_nodes,
                      VerifyReport, gpd_verify_decode, gpd_row_mean, gpd_sigmoid_bwd_sparse,
                      gpd_decode_static, gpd_timing_tag, gpd_timing_collect, gpd_timing_reset, gpd_mlp_step)
