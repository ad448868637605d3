"""CPU oracle (test infrastructure only): see oracle/decoder.py."""
