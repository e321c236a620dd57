"""Usage examples of the STL library (run on an MI355X)."""
