"""MI355X-native hot path of AgentSAM speculative decoding (one step over a batch of sessions)."""
