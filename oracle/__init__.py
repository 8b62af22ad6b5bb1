"""CPU oracle (test infrastructure).  Import `oracle.ds_oracle`."""
