"""fp64 CPU reference for the R-Part (test infrastructure only; see rpart_oracle.c)."""
