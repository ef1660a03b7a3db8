"""CPU oracle of the KV-swap path.  Test infrastructure only: see kv_oracle.py."""
