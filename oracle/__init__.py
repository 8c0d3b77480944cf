"""CPU fp64 oracle for Gradient Agreement Filtering. Test infrastructure only."""
