"""CPU oracle of the vote step: test infrastructure, not the product."""
