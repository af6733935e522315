"""CPU oracle of the clustered vocabulary projection: test infrastructure only."""
