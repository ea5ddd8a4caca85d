"""CPU oracle (test infrastructure only): the plain definition the GPU path is checked against."""
