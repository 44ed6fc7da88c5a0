"""CPU oracles (test infrastructure only): ``predictor`` (fp64 numpy) and ``anticipator``
(plain C).  Nothing in the product path may import this package."""
