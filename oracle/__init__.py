"""fp64 CPU oracle (test infrastructure only; see streaming_attention.py)."""
