"""Test and benchmark harness: seeded synthetic inputs and the error metric.  Not part of the product package."""
