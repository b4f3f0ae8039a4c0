"""CPU oracle of Ozaki scheme II: test infrastructure, not part of the product path."""
