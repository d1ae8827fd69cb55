"""AIS-GRPO hot path for MI355X (gfx950): token log-probs, AIS diagnostics, loss and dlogits."""
