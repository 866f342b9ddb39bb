"""Test-only CPU oracle; see rtp_oracle.py.  Never imported by the product path."""
