"""CPU oracle (test infrastructure).  See mixers.py and kv_layout.py."""
