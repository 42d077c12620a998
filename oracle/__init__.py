"""Test-only CPU oracle (see dare_oracle.py).  Never imported by the product."""
