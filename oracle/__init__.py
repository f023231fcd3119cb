"""fp64 CPU oracle for 2D Neighborhood Attention -- test infrastructure, not product code."""
