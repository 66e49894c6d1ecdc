"""CPU oracle of the PatternKV hot path.  Test infrastructure only."""
