"""CPU oracle of the AMS compression event.  Test infrastructure only."""
