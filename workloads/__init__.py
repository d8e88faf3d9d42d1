"""Seeded synthetic inputs (graphs, features, caches, parameters, chunk sets) for the tests, the
smoke run and the benchmark.  Not part of the product package: it only draws inputs and holds
none of the layer's arithmetic; the CPU oracle and the HIP path both read the arrays it returns."""
