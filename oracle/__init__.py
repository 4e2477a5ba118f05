"""CPU oracle of the Fed-CVLC compressor (test infrastructure only)."""
