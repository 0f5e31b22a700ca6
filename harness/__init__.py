"""Seeded synthetic inputs (graphs, id streams, initial tables) shared by the tests, the benchmark, the GPU
library's callers and the CPU oracle's callers.  Holds none of the method's arithmetic and imports neither
the GPU package nor the oracle."""
