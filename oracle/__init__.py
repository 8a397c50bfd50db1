"""CPU oracle (test infrastructure only; see fastcache_oracle.py)."""
