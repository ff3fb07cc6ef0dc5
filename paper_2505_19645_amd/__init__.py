"""MoE FFN layer forward for speculative-decoding verification batches on one
MI355X: a C-ABI HIP library (libmoesd.so, see include/moesd.h) and its ctypes
binding.  `synth` generates the seeded synthetic inputs."""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    LayerDesc, Weights, MoesdError, lib, make_desc, make_weights, moesd_expected_active_experts, moesd_expected_active_experts_p,
    moesd_expected_tokens_per_expert, moesd_moe_forward, moesd_moe_forward_static, moesd_permute, moesd_route,
    moesd_token_threshold, moesd_workspace_bytes, status_string, last_hip_error,
)
