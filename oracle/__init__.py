"""CPU checker package (test infrastructure only; the product never imports it)."""
