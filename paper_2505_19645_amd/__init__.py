"""MoE layer forward for speculative-decoding verification batches on MI355X."""
