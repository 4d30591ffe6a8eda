"""CPU oracle: test infrastructure only (see qg_oracle.c).  Never imported by the product."""
