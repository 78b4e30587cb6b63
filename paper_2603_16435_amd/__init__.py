"""MI355X-native fused LM-head log-prob + policy-loss (GRPO / flow-balance) path.

`synth` builds seeded synthetic rollout batches; `binding` marshals arguments into
the C-ABI library built from `csrc/` (loaded on first use; there is no fallback)."""
