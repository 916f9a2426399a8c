"""Float64 CPU oracle of the CoS verification step: test infrastructure only."""
