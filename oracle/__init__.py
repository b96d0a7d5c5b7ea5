"""CPU oracle package: test infrastructure only (see spiffy_oracle.py's header).
Nothing in the product imports this package."""
