"""CPU oracle of the NOVAK update step.  Test infrastructure only: never imported by the product."""
