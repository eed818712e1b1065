"""CPU oracle for the small-batch GeMM (test infrastructure only; never on the product path)."""
