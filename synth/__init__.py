"""Seeded synthetic inputs (weights, prompts, uniforms) shared by the CPU oracle's tests and the
HIP path's tests.  Holds data generation only: none of the method's arithmetic lives here."""
