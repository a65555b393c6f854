"""Plain CPU oracle of the re-attachment path.  Test infrastructure only."""
