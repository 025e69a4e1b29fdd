"""CPU oracle (test infrastructure).  Never imported by the product package."""
