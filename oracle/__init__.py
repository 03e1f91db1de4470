"""CPU oracle for Sliding Tile Attention.  Test infrastructure only: nothing
in the product package may import from here."""
