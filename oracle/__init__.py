"""CPU oracle: test infrastructure only (see ref.py and patdnn_ref.c)."""
