"""CPU oracle (test infrastructure only): see ht_oracle.py.  Never imported by the product path."""
