"""CPU oracle (test infrastructure).  See epd_oracle.py."""
