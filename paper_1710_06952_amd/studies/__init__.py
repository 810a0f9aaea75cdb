"""Small studies that drive the library with schedules of their own (no arithmetic of the method here)."""
