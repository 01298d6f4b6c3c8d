"""Float64 CPU oracle of AdaCons aggregation -- test infrastructure only."""
