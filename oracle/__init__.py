"""Plain CPU oracle of the EXEC hot path (test infrastructure, never imported by
the product package)."""
