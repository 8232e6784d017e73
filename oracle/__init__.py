"""Plain CPU oracle of the FB4 quantizer: test infrastructure, never a product path."""
