"""CPU oracle of the AdaTopK path.  Test infrastructure only: never imported by the product."""
