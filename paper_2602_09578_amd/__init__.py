"""MI355X-native rollout decode step: paged shared-prefix decode attention and per-token
log-probabilities behind a C ABI (see include/marl_decode.h)."""
