"""CPU oracle for the Speculative Thinking hot path.  Test infrastructure only."""
