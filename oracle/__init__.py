"""CPU oracle for the banded local-operator chain. Test infrastructure only:
nothing in the product package imports this."""
