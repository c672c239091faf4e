"""List-level Gumbel-max coupling (GLS) on MI355X: Python binding of the HIP library."""
