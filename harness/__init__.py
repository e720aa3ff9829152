"""Test and benchmark harness: seeded synthetic inputs.  Not part of the product package; holds none of the
method's arithmetic and imports neither the HIP binding nor the oracle."""
