"""Plain CPU oracle of the OSP synchronization step: test infrastructure only."""
