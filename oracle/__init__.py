"""CPU oracle of the InfiniGen rehearsal path. Test infrastructure only."""
