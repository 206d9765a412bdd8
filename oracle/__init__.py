"""Plain CPU oracle of the W4A8 linear layer.  Test infrastructure: imported only by tests, the
smoke check and the benchmark's cpu_baseline leg -- never by the product package."""
