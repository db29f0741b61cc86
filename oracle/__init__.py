"""CPU oracle (test infrastructure only; see kv_oracle.py and s3_oracle.c)."""
