"""MI355X-native Monte-Carlo simulator of the gate-and-route LLM-inference queueing network.

`workloads` and `plan` are host-side input preparation; `binding` (imported lazily)
wraps the C-ABI library built from `csrc/`.
"""
__all__ = ["workloads", "plan"]
