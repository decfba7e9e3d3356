"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side
harness.  Holds no arithmetic of the method itself."""
