"""Measurement aids behind the tile-size and occupancy decisions recorded under profiles/:
A/B timing of library variants (ab_time.py) and an instruction-issue microbenchmark
(issue_model.hip).  Nothing here is on the path the library's entry points take."""
