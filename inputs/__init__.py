"""Seeded synthetic input generators shared by the CPU oracle's tests and the GPU path's tests
and benchmark.  Inputs only: none of the layer's arithmetic lives here."""
