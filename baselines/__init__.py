"""Host-side comparison samplers for bench.py.  BASELINE / TEST INFRASTRUCTURE ONLY: imported by
tests/ and by bench.py's CPU legs, never by the product path, and not the oracle (that is oracle/)."""
