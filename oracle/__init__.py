"""CPU oracle for the Cascade-Speculative-Drafting verify path: test infrastructure only."""
